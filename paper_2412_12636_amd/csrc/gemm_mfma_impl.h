// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// A block of WGM x WGN wavefronts (four or eight) owns a BM x BN output tile and walks the reduction
// axis 64 elements at a time through two LDS stages.  (Four waves on a 256x192 tile own 128x96 each: fewer
// LDS bytes per MFMA, one wave per SIMD, accumulators in the upper half of the 512-register file.)
//
// Main kernel (gemm_pipe_kernel).  Operand tiles go from global memory STRAIGHT into LDS
// (buffer_load ... lds, 16 bytes per lane): no staging registers, no LDS store instructions.  A
// wave-wide load fills 1024 contiguous LDS bytes, so any layout permutation is applied on the
// global side: each lane fetches the 16-byte chunk that belongs at its LDS position.
//   * Operand with contiguous reduction axis (x and W in y = x W^T, dy in dx = dy W): LDS tile
//     [row][64], chunks XOR-swizzled by row; MFMA fragments are plain 16-byte LDS reads.
//   * Operand with strided reduction axis (W in dx = dy W; dy and x in dW = dy^T x): LDS tile
//     [k][rows], i.e. the global layout; MFMA fragments come from the transposing LDS read
//     ds_read_b64_tr_b16, which hands each lane four consecutive k of one row.  No transposed copies
//     in HBM, no register shuffles.
// The loads of step k+2 are issued during step k; one barrier per step, placed before the LAST 16-wide
// slice of the step so that the LDS reads and the global loads that follow it overlap that slice's MFMAs;
// the waits on the loads are explicit (s_waitcnt vmcnt), since the compiler does not track the LDS side of
// these loads.  With a grid of several block rows the kernel splits the reduction: block row y takes
// the y-th part of K and writes the y-th fp32 result (added up by the caller).
// What bounds the kernel is the path from L2 into LDS (about 50 bytes per clock and compute unit, and
// only whole 128-byte lines count: hence 64-element steps) together with the LDS reads, so the tile
// shapes trade traffic per flop against how evenly the tiles fill the 256 compute units.
// A reduction length that is not a multiple of 64 cannot be masked on this path; such shapes take the
// staged kernel below.
//
// Staged kernel (gemm_staged_kernel): 128x128 tile, global -> registers -> LDS with the reduction
// tail masked on the way; strided operands are transposed in registers.  Any K that is a multiple of 8.
//
// Global accesses use buffer descriptors: reads past the end of a tensor return zero and writes
// past the end are dropped, so ragged M / N edges need no branches.  Only the per-lane offset is
// checked against the descriptor's size, so everything that can run past the end travels in it.
//
// Epilogue.  bf16 results: the MFMA operands are passed swapped, so an accumulator tile is C^T and every
// lane owns four consecutive output columns of one row; the block's tile is assembled in LDS and leaves
// as whole rows (16 bytes per lane), a residual operand arrives the same way.  fp32 results: natural
// orientation, a store instruction writes two whole 128-byte lines, streamed past the caches.  (The staged
// kernel stores its bf16 results straight from the accumulators.)
//
// Block index -> tile mapping: consecutive hardware block ids land on different XCDs (8 per chip,
// each with its own L2); ids are re-numbered so that every XCD works on a contiguous range of
// tiles, with the M tiles of one weight column adjacent.
#pragma once
#include <string>

#include "gemm.h"

namespace tmk {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int v4u32 __attribute__((__vector_size__(16)));  // the buffer builtins' own vector type
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int NXCD = 8;
constexpr int GEMM_BK = 64;  // reduction elements per step: one 128-byte line per tile row

__device__ __forceinline__ u32x4 buf_load16(rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
}

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
  uint32_t a_bytes, b_bytes, c_bytes;  // extents of the tensors, for the buffer descriptors
  AdamTarget adam;                     // EPI 3 only
  int stagger_ticks, stagger_phases, stagger_blocks;  // EPI 3 only, see stagger_by_unit(); 0 ticks: off
};

// The fused-update product runs in two phases per tile: the main loop, which pulls operands through the compute unit's
// memory path at the rate that path allows, and the update, which streams 26 bytes per parameter of optimizer state
// and is bound by HBM when every unit of the chip streams at once.  With one large block per unit, launched together,
// all units are in the same phase: HBM idles during the main loops and is oversubscribed during the updates.  The
// first block on each unit is therefore held back by a delay that depends on the unit (its identity in the hardware
// registers: XCC, shader engine, array, unit): half of the units start one main loop late, so that at any time about
// half of the chip streams, at twice the share of HBM, while the other half multiplies.  Blocks that start later
// inherit the phase of the block whose place they take.  (With two small blocks per unit the same offsets gain
// nothing: that form is bound by the unit's memory path in both phases.)
__device__ __forceinline__ void stagger_by_unit(int ticks, int phases) {
  unsigned hw, xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID, 8, 8)" : "=s"(hw));  // cu_id [3:0], sh_id [4], se_id [7:5]
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(xcc));
  const unsigned phase = ((hw & 15) + (hw >> 4) + xcc) % (unsigned)phases;
  const uint64_t wait = (uint64_t)ticks * phase / (unsigned)phases, t0 = wall_clock64();
  while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(32);  // the clock only moves forward: ends
}

// Block id -> output tile.  Hardware block ids go round-robin over the 8 XCDs; ids are first
// re-numbered so that each XCD owns a contiguous range, then the range is walked in groups of
// GROUP_M row-tiles by all column-tiles, row-tile fastest.  The blocks an XCD runs at the same time
// then form a roughly square patch of tiles and share both operands' slices in that XCD's L2.
constexpr int GROUP_M = 8;
__device__ __forceinline__ void tile_of_block(const MfmaGemmParams &p, int BM, int BN, int &m0, int &n0) {
  const int nblk = gridDim.x, pid = blockIdx.x;
  const int xcd = pid % NXCD, local = pid / NXCD;
  const int base = nblk / NXCD, rem = nblk % NXCD;
  const int lid = xcd * base + (xcd < rem ? xcd : rem) + local;
  // 32 compute units of an XCD run a patch of gm x (tiles / gm) tiles at a time and fetch gm*BM + (tiles/gm)*BN operand
  // rows a step from memory (first touches in that XCD's L2; 20 % of the requests with 8 x 4 tiles of 256x192, 18 % with
  // 4 x 8): 8 row-tiles for the 128- and 192-row tiles (two blocks a unit), 4 for the 256-row tiles
  const int gm = BM >= 256 ? GROUP_M / 2 : GROUP_M;
  const int per_group = gm * p.tiles_n;
  const int group = lid / per_group, first_m = group * gm;
  const int gsz = p.tiles_m - first_m < gm ? p.tiles_m - first_m : gm;
  const int in_group = lid - group * per_group;
  m0 = (first_m + in_group % gsz) * BM;
  n0 = (in_group / gsz) * BN;
}

// ---- epilogue shared by both kernels -------------------------------------------------------------
// EPI 0: bf16 C = acc (+bias) (+residual); acc[i][j] is the transposed 32x32 tile (rows = output columns):
// register 4q+e of lane l holds C[row = .. + l%32][col = .. + 8q + 4*(l/32) + e].
// EPI 1: fp32 C += acc;  EPI 2: fp32 C = acc; acc[i][j] is the tile itself: register v of lane l holds
// C[row = .. + 8*(v/4) + 4*(l/32) + v%4][col = .. + l%32].
// bf16 results: operands swapped, the accumulator tile is C^T (lane = row, 4 consecutive columns per
// register quad: 8-byte stores).  fp32 results: natural order, the tile is C (lane%32 = column): a store
// instruction writes two whole 128-byte lines.
template <int EPI> __device__ __forceinline__ f32x16 mfma_for(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (EPI == 0) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// VB: accumulator registers of a 32x32 tile whose state reads are in flight together in the update epilogue (EPI 3):
// all sixteen where a wave has 256 registers, eight where three waves share a SIMD's register file
// The update of one 32x32 accumulator tile (EPI 3): register v of lane l holds the gradient of row row0 + 8(v/4) + 4hh + v%4,
// column col.  All 48 state reads of the tile are in flight together; gradient (if stored), state and the bf16 copy
// are streamed past the caches.
struct AdamRsrc {
  rsrc_t rc, rp, rm, rv, rl;
};
__device__ __forceinline__ AdamRsrc adam_rsrc(const MfmaGemmParams &p) {
  return AdamRsrc{make_rsrc(p.C, p.c_bytes), make_rsrc(p.adam.master, p.c_bytes), make_rsrc(p.adam.exp_avg, p.c_bytes),
                  make_rsrc(p.adam.exp_avg_sq, p.c_bytes), make_rsrc(p.adam.lowp, p.c_bytes / 2)};
}
__device__ __forceinline__ void adam_tile(const MfmaGemmParams &p, const AdamRsrc &r, const f32x16 &g, int row0, int col, int hh) {
  constexpr int kNonTemporal = 2;
  uint32_t off[16];
  float pw[16], mw[16], vw[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = row0 + 8 * (v >> 2) + 4 * hh + (v & 3);
    off[v] = col < p.N ? (uint32_t)(((int64_t)row * p.ldc + col) * 4) : 0xfffffff0u;
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    pw[v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r.rp, off[v], 0, kNonTemporal));
    mw[v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r.rm, off[v], 0, kNonTemporal));
    vw[v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r.rv, off[v], 0, kNonTemporal));
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const float gv = g[v];
    adam_one(pw[v], gv, mw[v], vw[v], p.adam.a);
    if (p.adam.store_grad)
      __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, gv), r.rc, off[v], 0, kNonTemporal);
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, pw[v]), r.rp, off[v], 0, kNonTemporal);
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, mw[v]), r.rm, off[v], 0, kNonTemporal);
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, vw[v]), r.rv, off[v], 0, kNonTemporal);
    const bf16 lo = (bf16)pw[v];
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, lo), r.rl,
                                          off[v] != 0xfffffff0u ? off[v] >> 1 : 0xfffffff0u, 0, kNonTemporal);
  }
}

#ifndef TM_LDW_VB
#define TM_LDW_VB 12
#endif
template <int TM, int TN, int EPI, int VB = 16>
__device__ __forceinline__ void epilogue(const MfmaGemmParams &p, const f32x16 (&acc)[TM][TN], int row_base,
                                         int col_base, int l32, int hh) {
  if constexpr (EPI == 3) {
    // weight gradient with the Adam update of its parameters: per accumulator register (two whole 128-byte
    // lines per wave) the three state reads are in flight together; gradient, state and the bf16 copy are
    // streamed past the caches
    constexpr int kNonTemporal = 2;
    const rsrc_t rc = make_rsrc(p.C, p.c_bytes);
    const rsrc_t rp = make_rsrc(p.adam.master, p.c_bytes), rm = make_rsrc(p.adam.exp_avg, p.c_bytes);
    const rsrc_t rv = make_rsrc(p.adam.exp_avg_sq, p.c_bytes), rl = make_rsrc(p.adam.lowp, p.c_bytes / 2);
    constexpr int NACC = TM * TN * 16;  // the wave's accumulator registers, walked tile by tile in batches of VB
    static_assert(NACC % VB == 0, "whole batches");
#pragma unroll
    for (int f0 = 0; f0 < NACC; f0 += VB) {
      uint32_t off[VB];
      float pw[VB], mw[VB], vw[VB];
#pragma unroll
      for (int u = 0; u < VB; ++u) {
        const int f = f0 + u, i = f / (TN * 16), j = (f / 16) % TN, v = f % 16;
        const int col = col_base + j * 32 + l32;
        const int row = row_base + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
        off[u] = col < p.N ? (uint32_t)(((int64_t)row * p.ldc + col) * 4) : 0xfffffff0u;
      }
#pragma unroll
      for (int u = 0; u < VB; ++u) {
        pw[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rp, off[u], 0, kNonTemporal));
        mw[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rm, off[u], 0, kNonTemporal));
        vw[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, off[u], 0, kNonTemporal));
      }
#pragma unroll
      for (int u = 0; u < VB; ++u) {
        const int f = f0 + u;
        const float g = acc[f / (TN * 16)][(f / 16) % TN][f % 16];
        adam_one(pw[u], g, mw[u], vw[u], p.adam.a);
        if (p.adam.store_grad)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, g), rc, off[u], 0, kNonTemporal);
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, pw[u]), rp, off[u], 0, kNonTemporal);
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, mw[u]), rm, off[u], 0, kNonTemporal);
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, vw[u]), rv, off[u], 0, kNonTemporal);
        const bf16 lo = (bf16)pw[u];
        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, lo), rl,
                                              off[u] != 0xfffffff0u ? off[u] >> 1 : 0xfffffff0u, 0, kNonTemporal);
      }
    }
    return;
  }
  if constexpr (EPI != 0) {
    // fp32 results (weight gradients): whole lines, written once and next read by the optimizer: streamed
    // past the caches, which keeps the operands of the following products resident
    constexpr int kStoreNonTemporal = 2;  // cache-policy operand of the buffer store: the nt bit
    const rsrc_t rc = make_rsrc(p.C, p.c_bytes);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col_base + j * 32 + l32;
        const bool col_ok = col < p.N;
        uint32_t off[16];
        float old[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row_base + i * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
          off[v] = col_ok ? (uint32_t)(((int64_t)row * p.ldc + col) * 4) : 0xfffffff0u;
        }
        if (EPI == 1) {  // all sixteen reads of the tile are in flight before the first add
#pragma unroll
          for (int v = 0; v < 16; ++v)
            old[v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rc, off[v], 0, kStoreNonTemporal));
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float o = EPI == 1 ? old[v] + acc[i][j][v] : acc[i][j][v];
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, o), rc, off[v], 0, kStoreNonTemporal);
        }
      }
    return;
  }
  const uint32_t c_elem = 2u;
  const rsrc_t rc = make_rsrc(p.C, p.c_bytes);
  const rsrc_t rres = make_rsrc(p.residual ? (const void *)p.residual : p.C, p.c_bytes);
  const rsrc_t rbias = make_rsrc(p.bias ? (const void *)p.bias : p.C, (uint32_t)p.N * 2u);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int col = col_base + j * 32 + 8 * q + 4 * hh;
      const bool col_ok = col < p.N;  // N is a multiple of 8: the four columns are in or out together
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (EPI == 0 && p.bias) {
        const u32x2 braw = __builtin_bit_cast(
            u32x2, __builtin_amdgcn_raw_buffer_load_b64(rbias, col_ok ? (uint32_t)col * 2u : 0xfffffff0u, 0, 0));
        bv[0] = __builtin_bit_cast(float, braw[0] << 16);
        bv[1] = __builtin_bit_cast(float, braw[0] & 0xffff0000u);
        bv[2] = __builtin_bit_cast(float, braw[1] << 16);
        bv[3] = __builtin_bit_cast(float, braw[1] & 0xffff0000u);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = row_base + i * 32 + l32;
        const uint32_t off = col_ok ? (uint32_t)(((int64_t)row * p.ldc + col) * c_elem) : 0xfffffff0u;
        {
          float r[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) r[e] = acc[i][j][4 * q + e] + bv[e];
          if (p.residual) {
            const u32x2 rr = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rres, off, 0, 0));
            r[0] += __builtin_bit_cast(float, rr[0] << 16);
            r[1] += __builtin_bit_cast(float, rr[0] & 0xffff0000u);
            r[2] += __builtin_bit_cast(float, rr[1] << 16);
            r[3] += __builtin_bit_cast(float, rr[1] & 0xffff0000u);
          }
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)r[e];
          __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, o), rc, off, 0, 0);
        }
      }
    }
  }
}

// =================================================================================================
// direct-to-LDS kernel
// =================================================================================================

// ---- operand with contiguous reduction axis: element (r, k) at base[r*ld + k]; LDS [R][BK] --------
template <int R, int BK, int NW = 4> struct DirectKC {
  static constexpr int ROWB = BK * 2;               // bytes per LDS row
  static constexpr int CPR = BK / 8;                // 16-byte chunks per row
  static constexpr int RPL = 64 / CPR;              // rows covered by one wave-wide load
  static constexpr int NLOAD = R / (NW * RPL);      // loads per wave and step
  static_assert(R % (NW * RPL) == 0, "rows per load");
  static constexpr int BYTES = R * ROWB;
  // rows that are 8 apart in a fragment read must not share banks: XOR the chunk index with low row bits
  static __device__ __forceinline__ int swz(int row) {
    return BK == 64 ? ((row ^ (row >> 3)) & 7) : ((row >> 1) & 3);
  }
  uint32_t voff[NLOAD];
  __device__ __forceinline__ void init(int64_t ld, int row0, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int row = (i * NW + wave) * RPL + lane / CPR;
      const int c = (lane % CPR) ^ swz(row);  // logical chunk that belongs at this lane's LDS position
      voff[i] = (uint32_t)(((int64_t)(row0 + row) * ld + c * 8) * 2);
    }
  }
  __device__ __forceinline__ void issue(rsrc_t rs, char *tile, int k0, int64_t /*ld*/, int wave) const {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, voff[i],
                                               (uint32_t)k0 * 2u, 0, 0);
  }
  // fragment of the 32-row block starting at r32: lane's row r32 + lane%32, reduction slots 16ks + 8hh + 0..7
  static __device__ __forceinline__ bf16x8 frag(const char *tile, int r32, int ks, int lane) {
    const int r = r32 + (lane & 31), hh = lane >> 5;
    return *reinterpret_cast<const bf16x8 *>(tile + r * ROWB + (((2 * ks + hh) ^ swz(r)) << 4));
  }
};

// ---- operand with strided reduction axis: element (r, k) at base[k*ld + r]; LDS [BK][R] ------------
template <int R, int BK, int NW = 4> struct DirectKS {
  static constexpr int ROWB = R * 2;                // bytes per LDS k-row
  static constexpr int CPR = R / 8;                 // chunks per k-row (32 or 16)
  static constexpr int NLOAD = BK * CPR / (64 * NW);  // loads per wave and step
  static_assert((BK * CPR) % (64 * NW) == 0, "chunks per load");
  static constexpr int BYTES = BK * ROWB;
  // The transposing read of a 16-lane group touches 4 k-rows x 32 contiguous bytes, a half-wave the
  // neighbouring 32 bytes as well; k-rows alias in the banks (row pitch 256/512 bytes).  The position
  // of chunk c in k-row kk spreads the four k-rows over distinct 32-byte windows and sends the
  // neighbouring group to the other 128-byte half.
  // (With 24 chunks per k-row the row pitch is 384 bytes, consecutive k-rows already differ by 128 bytes,
  // and the XOR of bits 2:1 alone separates everything.)
  static __device__ __forceinline__ int place(int c, int kk) {
    return CPR % 16 == 0 ? c ^ (((kk & 3) << 1) | (((c >> 1) & 1) << 3)) : c ^ ((kk & 3) << 1);
  }
  static __device__ __forceinline__ int unplace(int pc, int kk) {
    const int low = pc ^ ((kk & 3) << 1);           // bits 2:1 restored
    return CPR % 16 == 0 ? low ^ (((low >> 1) & 1) << 3) : low;
  }
  uint32_t voff[NLOAD];
  __device__ __forceinline__ void init(int64_t ld, int row0, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int idx = (i * NW + wave) * 64 + lane;
      const int kk = idx / CPR, c = unplace(idx % CPR, kk);
      voff[i] = (uint32_t)(((int64_t)kk * ld + row0 + c * 8) * 2);
    }
  }
  __device__ __forceinline__ void issue(rsrc_t rs, char *tile, int k0, int64_t ld, int wave) const {
    // the step offset travels in the per-lane offset: that one is checked against the buffer size
    const uint32_t koff = (uint32_t)((int64_t)k0 * ld * 2);
#pragma unroll
    for (int i = 0; i < NLOAD; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)(tile + (i * NW + wave) * 1024), 16, voff[i] + koff, 0, 0, 0);
  }
  // ds_read_b64_tr_b16: within 16 lanes, lane i receives element (i%4) of the 8-byte pieces addressed
  // by lanes i/4, i/4+4, i/4+8, i/4+12.  With lane s addressing T[k0 + s/4][r0 + 4*(s%4) ..+3], lane i
  // ends up with T[k0 .. k0+3][r0 + i]: four consecutive k of one row.
  static __device__ __forceinline__ bf16x8 frag(const char *tile, int r32, int ks, int lane) {
    const int g = lane >> 4, s = lane & 15;
    const int r = r32 + 16 * (g & 1) + 4 * (s & 3);
    const int c = r >> 3, half = (r >> 2) & 1;
    union { s16x4 h[2]; bf16x8 v; } x;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kk = 16 * ks + 8 * (g >> 1) + 4 * t + (s >> 2);
      const char *a = tile + kk * ROWB + (place(c, kk) << 4) + (half << 3);
      x.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(a));
    }
    return x.v;
  }
};

template <int R, int BK, bool KC, int NW = 4> struct DirectSel { typedef DirectKC<R, BK, NW> type; };
template <int R, int BK, int NW> struct DirectSel<R, BK, false, NW> { typedef DirectKS<R, BK, NW> type; };

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// ---- bf16 epilogue through LDS --------------------------------------------------------------------
// The accumulator layout gives every lane 8 bytes in each of many rows; written to global memory directly
// that is 32 partial lines per store instruction.  Instead the block's tile is assembled in LDS (the
// stages are free after the main loop) and leaves as whole rows, 16 bytes per lane; a residual operand
// comes in the same way.  The arithmetic is unchanged: acc + bias + residual in fp32, one rounding.
// Position of 16-byte chunk c of tile row `row`: XOR with low row bits, so that the 8-byte accesses of 32
// consecutive rows spread over all banks.
template <int CPR> __device__ __forceinline__ int epi_place(int c, int row) {
  if (c < (CPR & ~15)) return (c & ~15) | ((c ^ row) & 15);
  return (c & ~7) | ((c ^ row) & 7);
}
template <int BM, int BN, int NW, int TM, int TN>
__device__ __forceinline__ void epilogue_lds(const MfmaGemmParams &p, const f32x16 (&acc)[TM][TN], char *lds, int m0,
                                             int n0, int wrow, int wcol, int lane) {
  constexpr int CPR = BN / 8, ROWB = BN * 2, NT = 64 * NW, CHUNKS = BM * CPR;
  static_assert(CHUNKS % NT == 0, "whole passes");
  const int l32 = lane & 31, hh = lane >> 5, tid = threadIdx.x;
  const rsrc_t rc = make_rsrc(p.C, p.c_bytes);
  if (p.residual) {
    const rsrc_t rres = make_rsrc(p.residual, p.c_bytes);
#pragma unroll
    for (int it = 0; it < CHUNKS / NT; ++it) {
      const int idx = it * NT + tid, row = idx / CPR, c = idx % CPR;
      const int gcol = n0 + c * 8;
      const uint32_t off = gcol < p.N ? (uint32_t)(((int64_t)(m0 + row) * p.ldc + gcol) * 2) : 0xfffffff0u;
      const u32x4 v = buf_load16(rres, off, 0);
      *reinterpret_cast<u32x4 *>(lds + row * ROWB + (epi_place<CPR>(c, row) << 4)) = v;
    }
    __syncthreads();
  }
  const rsrc_t rbias = make_rsrc(p.bias ? (const void *)p.bias : p.C, (uint32_t)p.N * 2u);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int tcol = wcol + j * 32 + 8 * q + 4 * hh;  // column inside the tile
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (p.bias) {
        const int col = n0 + tcol;
        const u32x2 braw = __builtin_bit_cast(
            u32x2, __builtin_amdgcn_raw_buffer_load_b64(rbias, col < p.N ? (uint32_t)col * 2u : 0xfffffff0u, 0, 0));
        bv[0] = __builtin_bit_cast(float, braw[0] << 16);
        bv[1] = __builtin_bit_cast(float, braw[0] & 0xffff0000u);
        bv[2] = __builtin_bit_cast(float, braw[1] << 16);
        bv[3] = __builtin_bit_cast(float, braw[1] & 0xffff0000u);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wrow + i * 32 + l32;
        char *at = lds + row * ROWB + (epi_place<CPR>(tcol >> 3, row) << 4) + ((tcol & 4) << 1);
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = acc[i][j][4 * q + e] + bv[e];
        if (p.residual) {
          const u32x2 rr = *reinterpret_cast<const u32x2 *>(at);
          r[0] += __builtin_bit_cast(float, rr[0] << 16);
          r[1] += __builtin_bit_cast(float, rr[0] & 0xffff0000u);
          r[2] += __builtin_bit_cast(float, rr[1] << 16);
          r[3] += __builtin_bit_cast(float, rr[1] & 0xffff0000u);
        }
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)r[e];
        *reinterpret_cast<bf16x4 *>(at) = o;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < CHUNKS / NT; ++it) {
    const int idx = it * NT + tid, row = idx / CPR, c = idx % CPR;
    const int gcol = n0 + c * 8;
    const uint32_t off = gcol < p.N ? (uint32_t)(((int64_t)(m0 + row) * p.ldc + gcol) * 2) : 0xfffffff0u;
    const u32x4 v = *reinterpret_cast<const u32x4 *>(lds + row * ROWB + (epi_place<CPR>(c, row) << 4));
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u32, v), rc, off, 0, 0);
  }
}

// The same epilogue in pieces, for blocks in which only some waves hold accumulators: all NW waves copy the
// residual in (residual_in) or the finished tile out, the accumulator waves add in between.
template <int BM, int BN, int NW>
__device__ __forceinline__ void epilogue_lds_copy(const MfmaGemmParams &p, char *lds, int m0, int n0, bool residual_in) {
  constexpr int CPR = BN / 8, ROWB = BN * 2, NT = 64 * NW, CHUNKS = BM * CPR;
  if (residual_in && !p.residual) return;
  const int tid = threadIdx.x;
  const rsrc_t rg = make_rsrc(residual_in ? (const void *)p.residual : (const void *)p.C, p.c_bytes);
#pragma unroll
  for (int it = 0; it < (CHUNKS + NT - 1) / NT; ++it) {
    const int idx = it * NT + tid, row = idx / CPR, c = idx % CPR;
    if (CHUNKS % NT != 0 && idx >= CHUNKS) break;  // the last pass may be ragged
    const int gcol = n0 + c * 8;
    const uint32_t off = gcol < p.N ? (uint32_t)(((int64_t)(m0 + row) * p.ldc + gcol) * 2) : 0xfffffff0u;
    char *at = lds + row * ROWB + (epi_place<CPR>(c, row) << 4);
    if (residual_in) {
      *reinterpret_cast<u32x4 *>(at) = buf_load16(rg, off, 0);
    } else {
      const u32x4 v = *reinterpret_cast<const u32x4 *>(at);
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u32, v), rg, off, 0, 0);
    }
  }
}
template <int BM, int BN, int TM, int TN>
__device__ __forceinline__ void epilogue_lds_acc(const MfmaGemmParams &p, const f32x16 (&acc)[TM][TN], char *lds, int n0,
                                                 int wrow, int wcol, int lane) {
  constexpr int CPR = BN / 8, ROWB = BN * 2;
  const int l32 = lane & 31, hh = lane >> 5;
  const rsrc_t rbias = make_rsrc(p.bias ? (const void *)p.bias : p.C, (uint32_t)p.N * 2u);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int tcol = wcol + j * 32 + 8 * q + 4 * hh;  // column inside the tile
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (p.bias) {
        const int col = n0 + tcol;
        const u32x2 braw = __builtin_bit_cast(
            u32x2, __builtin_amdgcn_raw_buffer_load_b64(rbias, col < p.N ? (uint32_t)col * 2u : 0xfffffff0u, 0, 0));
        bv[0] = __builtin_bit_cast(float, braw[0] << 16);
        bv[1] = __builtin_bit_cast(float, braw[0] & 0xffff0000u);
        bv[2] = __builtin_bit_cast(float, braw[1] << 16);
        bv[3] = __builtin_bit_cast(float, braw[1] & 0xffff0000u);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wrow + i * 32 + l32;
        char *at = lds + row * ROWB + (epi_place<CPR>(tcol >> 3, row) << 4) + ((tcol & 4) << 1);
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = acc[i][j][4 * q + e] + bv[e];
        if (p.residual) {
          const u32x2 rr = *reinterpret_cast<const u32x2 *>(at);
          r[0] += __builtin_bit_cast(float, rr[0] << 16);
          r[1] += __builtin_bit_cast(float, rr[0] & 0xffff0000u);
          r[2] += __builtin_bit_cast(float, rr[1] << 16);
          r[3] += __builtin_bit_cast(float, rr[1] & 0xffff0000u);
        }
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)r[e];
        *reinterpret_cast<bf16x4 *>(at) = o;
      }
    }
  }
}

// =================================================================================================
// pipelined kernel: WGM x WGN waves, two LDS stages, the barrier sits before the LAST reduction slice
// =================================================================================================
// Per step: slices 0..KS-2 run MFMAs while the LDS reads of the next slice are in flight.  Before the
// last slice every wave has read all it needs from the current stage and waits for its own loads of the
// next stage; after the barrier the current stage may be overwritten (loads of step kt+2) and the next
// stage may be read (its slice 0), and both overlap the MFMAs of the last slice, whose operands are
// already in registers.  No LDS latency is exposed behind the barrier.
// Issue order handed to the instruction scheduler, built at compile time (the builtin wants literal
// constants).  Masks: 0x008 MFMA, 0x020 global/buffer load, 0x100 LDS read.
template <int MASK, int N> __device__ __forceinline__ void sg() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
template <int MF, int DSN, int i> __device__ __forceinline__ void sched_mid() {
  if constexpr (i < MF) {
    sg<0x008, 1>();
    sg<0x100, DSN * (i + 1) / MF - DSN * i / MF>();
    sched_mid<MF, DSN, i + 1>();
  }
}
template <int MF, int DSN, int LOADS, int i> __device__ __forceinline__ void sched_last() {
  if constexpr (i < MF) {
    sg<0x008, 1>();
    sg<0x020, LOADS * (i + 1) / MF - LOADS * i / MF>();
    sg<0x100, DSN * (i + 1) / MF - DSN * i / MF>();
    sched_last<MF, DSN, LOADS, i + 1>();
  }
}

// NSA, NSB: LDS stages of the A and of the B tiles.  Two each is the base form.  A third stage lets a tile's loads
// be issued one step earlier (two steps of time to arrive instead of one): what bounds this kernel is the data it
// can have in flight between L2 and LDS (free LDS space) against the latency of that path (a 64 KB burst of a
// block takes about 2500 clocks to arrive even from L2), not LDS or MFMA throughput.  A third stage for B alone
// measured nothing (the A tiles of the same batch are as late); three of both need tiles of at most 53 KB a stage.
template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int EPI, int NSA = 2, int NSB = 2>
__global__ __launch_bounds__(64 * WGM * WGN, (WGM * WGN == 4 && BM * BN <= 256 * 128 && NSB == 2) ? 2 : 1) void gemm_pipe_kernel(
    const MfmaGemmParams p_in) {
  static_assert(NSA >= 2 && NSA <= 3 && NSB >= NSA && NSB <= 3, "two or three LDS stages, B at least as many as A");
  extern __shared__ __align__(16) char lds[];
  MfmaGemmParams p = p_in;
  if (gridDim.y > 1) {  // split reduction: this block row takes one part of K and writes its own result
    const int part = p.K / (int)gridDim.y, first = (int)blockIdx.y * part;
    const int64_t a_skip = A_KC ? (int64_t)first : (int64_t)first * p.lda;
    const int64_t b_skip = B_KC ? (int64_t)first : (int64_t)first * p.ldb;
    p.A += a_skip;
    p.B += b_skip;
    p.a_bytes -= (uint32_t)(a_skip * 2);
    p.b_bytes -= (uint32_t)(b_skip * 2);
    p.K = part;
    p.C = (char *)p.C + (size_t)blockIdx.y * p.c_bytes;
  }
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
  typedef typename DirectSel<BM, BK, A_KC, NW>::type LA;
  typedef typename DirectSel<BN, BK, B_KC, NW>::type LB;
  constexpr int B_BASE = NSA * LA::BYTES;  // LDS: the A stages, then the B stages
  constexpr int LOADS = LA::NLOAD + LB::NLOAD;
  // loads that may still be in flight when step kt+1's tiles must have landed: the batches issued later
  constexpr int PENDING = (NSA - 2) * LA::NLOAD + (NSB - 2) * LB::NLOAD;
  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "fragment buffers alternate");
  constexpr int MF = TM * TN;
  constexpr int DSN = TM * (A_KC ? 1 : 2) + TN * (B_KC ? 1 : 2);

  int m0, n0;
  tile_of_block(p, BM, BN, m0, n0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  LA la;
  LB lb;
  const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
  la.init(p.lda, m0, wave, lane);
  lb.init(p.ldb, n0, wave, lane);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  bf16x8 a[2][TM], b[2][TN];
  // prologue: stage 0 in LDS, its slice 0 in registers, stage 1 in flight
  la.issue(ra, lds, 0, p.lda, wave);
  lb.issue(rb, lds + B_BASE, 0, p.ldb, wave);
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int i = 0; i < TM; ++i) a[0][i] = LA::frag(lds, wm * WM + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) b[0][j] = LB::frag(lds + B_BASE, wn * WN + j * 32, 0, lane);
#pragma unroll
  for (int ahead = 1; ahead < NSB; ++ahead) {
    const int k1 = (ahead < nk ? ahead : nk - 1) * BK;  // never past K: a surplus fetch repeats the last step
    if (ahead < NSA) la.issue(ra, lds + ahead * LA::BYTES, k1, p.lda, wave);
    lb.issue(rb, lds + B_BASE + ahead * LB::BYTES, k1, p.ldb, wave);
  }

  int ca = 0, na = 1, cb = 0, nb = 1;  // LDS stages of steps kt and kt+1, per operand
  for (int kt = 0; kt < nk; ++kt) {
    char *As = lds + ca * LA::BYTES;
    char *Bs = lds + B_BASE + cb * LB::BYTES;
    char *An = lds + na * LA::BYTES;
    char *Bn = lds + B_BASE + nb * LB::BYTES;
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) a[(ks + 1) & 1][i] = LA::frag(As, wm * WM + i * 32, ks + 1, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) b[(ks + 1) & 1][j] = LB::frag(Bs, wn * WN + j * 32, ks + 1, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = mfma_for<EPI>(a[ks & 1][i], b[ks & 1][j], acc[i][j]);
      sched_mid<MF, DSN, 0>();
    }
    __builtin_amdgcn_sched_barrier(0);
    // all reads of the current stages are complete, and this wave's loads of the next stages have landed (loads
    // complete in order; a batch is the A loads, then the B loads, so what may still be in flight of a three-deep
    // operand are the loads issued last)
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(PENDING) : "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // the current stages are free: fetch steps kt+NSA / kt+NSB into them (at the end the last step again, never consumed)
    la.issue(ra, As, (kt + NSA < nk ? kt + NSA : nk - 1) * BK, p.lda, wave);
    lb.issue(rb, Bs, (kt + NSB < nk ? kt + NSB : nk - 1) * BK, p.ldb, wave);
#pragma unroll
    for (int i = 0; i < TM; ++i) a[0][i] = LA::frag(An, wm * WM + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) b[0][j] = LB::frag(Bn, wn * WN + j * 32, 0, lane);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = mfma_for<EPI>(a[(KS - 1) & 1][i], b[(KS - 1) & 1][j], acc[i][j]);
    sched_last<MF, DSN, LOADS, 0>();
    ca = na;
    na = na + 1 == NSA ? 0 : na + 1;
    cb = nb;
    nb = nb + 1 == NSB ? 0 : nb + 1;
  }
  wait_vmcnt<0>();  // drain the look-ahead loads before the block may exit
  if constexpr (EPI == 0) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();  // every wave's loads have landed and its LDS reads are done: the stages are free
    epilogue_lds<BM, BN, NW, TM, TN>(p, acc, lds, m0, n0, wm * WM, wn * WN, lane);
  } else {
    epilogue<TM, TN, EPI>(p, acc, m0 + wm * WM, n0 + wn * WN, lane & 31, lane >> 5);
  }
}

// =================================================================================================
// kernel with loader waves: WGM x WGN waves multiply, NP more waves do nothing but fetch
// =================================================================================================
// A wave issues its instructions in order, and a global -> LDS load can only be issued while the memory pipeline
// has room for it: a whole 64 KB stage goes through that pipeline at about 45 bytes per clock, so a wave that has
// to issue its share of a stage between two MFMAs stands still for hundreds of clocks, and its MFMAs with it
// (time stamps inside the pipelined kernel: the slice of a step that carries the loads takes 1100 clocks for 380
// clocks of MFMA work).  Here the waves that multiply never issue a global load.  They read fragments and issue
// MFMAs; NP extra waves (one per SIMD) issue all the loads of a step right after the step's barrier and then wait
// for them, and the SIMD's issue logic serves the multiplying waves while a loader wave is held up.  Two LDS stages
// and the same barrier placement as the pipelined kernel (before the last reduction slice of a step), so an output
// element is accumulated in the same order as in every other configuration.
template <int BM, int BN, int BK, int WGM, int WGN, int NP, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(64 * (WGM * WGN + NP), 3) void gemm_ldw_kernel(const MfmaGemmParams p_in) {
  extern __shared__ __align__(16) char lds[];
  MfmaGemmParams p = p_in;
  if constexpr (EPI == 3) {
    if (p_in.stagger_ticks > 0 && (int)blockIdx.x < p_in.stagger_blocks) stagger_by_unit(p_in.stagger_ticks, p_in.stagger_phases);
  }
  if (gridDim.y > 1) {  // split reduction: this block row takes one part of K and writes its own result
    const int part = p.K / (int)gridDim.y, first = (int)blockIdx.y * part;
    const int64_t a_skip = A_KC ? (int64_t)first : (int64_t)first * p.lda;
    const int64_t b_skip = B_KC ? (int64_t)first : (int64_t)first * p.ldb;
    p.A += a_skip;
    p.B += b_skip;
    p.a_bytes -= (uint32_t)(a_skip * 2);
    p.b_bytes -= (uint32_t)(b_skip * 2);
    p.K = part;
    p.C = (char *)p.C + (size_t)blockIdx.y * p.c_bytes;
  }
  constexpr int NC = WGM * WGN;  // multiplying waves
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
  typedef typename DirectSel<BM, BK, A_KC, NP>::type LA;  // the tiles are fetched by the NP loader waves
  typedef typename DirectSel<BN, BK, B_KC, NP>::type LB;
  constexpr int B_BASE = 2 * LA::BYTES;
  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "fragment buffers alternate");
  constexpr int MF = TM * TN;
  constexpr int DSN = TM * (A_KC ? 1 : 2) + TN * (B_KC ? 1 : 2);
  // EPI 3 with eight multiplying waves and four loaders: HAND accumulator tiles per multiplying wave are updated by the loaders
  constexpr int HAND = 2;
  constexpr bool HANDOFF = EPI == 3 && NC == 8 && NP == 4 && MF == 6 && NC * HAND * 16 * 64 * 4 <= 2 * (BM + BN) * BK * 2;

  int m0, n0;
  tile_of_block(p, BM, BN, m0, n0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nk = (p.K + BK - 1) / BK;

  if (wave >= NC) {
    // ---- loader wave: stage 0, barrier, stage 1; then per step: wait for step kt+1, barrier, fetch step kt+2 ----
    const int lw = wave - NC;
    LA la;
    LB lb;
    const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
    la.init(p.lda, m0, lw, lane);
    lb.init(p.ldb, n0, lw, lane);
    la.issue(ra, lds, 0, p.lda, lw);
    lb.issue(rb, lds + B_BASE, 0, p.ldb, lw);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    {
      const int k1 = (1 < nk ? 1 : nk - 1) * BK;  // never past K: a surplus fetch repeats the last step
      la.issue(ra, lds + LA::BYTES, k1, p.lda, lw);
      lb.issue(rb, lds + B_BASE + LB::BYTES, k1, p.ldb, lw);
    }
    for (int kt = 0; kt < nk; ++kt) {
      wait_vmcnt<0>();  // this wave's part of step kt+1 has landed
      __builtin_amdgcn_s_barrier();
      const int k2 = (kt + 2 < nk ? kt + 2 : nk - 1) * BK;
      la.issue(ra, lds + (kt & 1) * LA::BYTES, k2, p.lda, lw);
      lb.issue(rb, lds + B_BASE + (kt & 1) * LB::BYTES, k2, p.ldb, lw);
    }
    wait_vmcnt<0>();  // drain the look-ahead loads before the stages are reused or the block exits
    if constexpr (EPI == 0) {
      __syncthreads();
      epilogue_lds_copy<BM, BN, NC + NP>(p, lds, m0, n0, /*residual_in=*/true);
      __syncthreads();  // the multiplying waves add their accumulators in between
      __syncthreads();
      epilogue_lds_copy<BM, BN, NC + NP>(p, lds, m0, n0, /*residual_in=*/false);
    }
    if constexpr (HANDOFF) {
      // the update of a third of the tile: two of every multiplying wave's six accumulator tiles come through LDS, so
      // that all twelve waves of the block stream optimizer state
      __syncthreads();  // the stages are free
      __syncthreads();  // the accumulator tiles are in LDS
      const AdamRsrc r = adam_rsrc(p);
      const float *h = reinterpret_cast<const float *>(lds);
#pragma unroll
      for (int q = 0; q < HAND * NC / NP; ++q) {
        const int slot = lw * (HAND * NC / NP) + q, cw = slot / HAND, f = MF - HAND + slot % HAND;
        const int i = f / TN, j = f % TN;
        f32x16 gacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) gacc[v] = h[(slot * 16 + v) * 64 + lane];
        adam_tile(p, r, gacc, m0 + (cw / WGN) * WM + i * 32, n0 + (cw % WGN) * WN + j * 32 + (lane & 31), lane >> 5);
      }
    }
    return;
  }

  // ---- multiplying wave ----
  const int wm = wave / WGN, wn = wave % WGN;
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  bf16x8 a[2][TM], b[2][TN];
  __builtin_amdgcn_s_barrier();  // stage 0 is in LDS
#pragma unroll
  for (int i = 0; i < TM; ++i) a[0][i] = LA::frag(lds, wm * WM + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) b[0][j] = LB::frag(lds + B_BASE, wn * WN + j * 32, 0, lane);
  __builtin_amdgcn_s_setprio(1);
  for (int kt = 0; kt < nk; ++kt) {
    const char *As = lds + (kt & 1) * LA::BYTES;
    const char *Bs = lds + B_BASE + (kt & 1) * LB::BYTES;
    const char *An = lds + ((kt + 1) & 1) * LA::BYTES;
    const char *Bn = lds + B_BASE + ((kt + 1) & 1) * LB::BYTES;
#pragma unroll
    for (int ks = 0; ks + 1 < KS; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) a[(ks + 1) & 1][i] = LA::frag(As, wm * WM + i * 32, ks + 1, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) b[(ks + 1) & 1][j] = LB::frag(Bs, wn * WN + j * 32, ks + 1, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma_for<EPI>(a[ks & 1][i], b[ks & 1][j], acc[i][j]);
      sched_mid<MF, DSN, 0>();
    }
    __builtin_amdgcn_sched_barrier(0);
    // every read of the current stage is complete; past the barrier the loaders overwrite it, and the next stage
    // (complete: the loaders waited for it) may be read
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TM; ++i) a[0][i] = LA::frag(An, wm * WM + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) b[0][j] = LB::frag(Bn, wn * WN + j * 32, 0, lane);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = mfma_for<EPI>(a[(KS - 1) & 1][i], b[(KS - 1) & 1][j], acc[i][j]);
    sched_last<MF, DSN, 0, 0>();
  }
  __builtin_amdgcn_s_setprio(0);
  if constexpr (EPI == 0) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();  // the loaders' last loads have landed and every fragment read is done: the stages are free
    epilogue_lds_copy<BM, BN, NC + NP>(p, lds, m0, n0, /*residual_in=*/true);
    __syncthreads();
    epilogue_lds_acc<BM, BN, TM, TN>(p, acc, lds, n0, wm * WM, wn * WN, lane);
    __syncthreads();
    epilogue_lds_copy<BM, BN, NC + NP>(p, lds, m0, n0, /*residual_in=*/false);
  } else if constexpr (HANDOFF) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();  // the loaders' last loads have landed and every fragment read is done: the stages are free
    float *h = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int t = 0; t < HAND; ++t) {
      const int f = MF - HAND + t, slot = wave * HAND + t;
#pragma unroll
      for (int v = 0; v < 16; ++v) h[(slot * 16 + v) * 64 + lane] = acc[f / TN][f % TN][v];
    }
    __syncthreads();
    const AdamRsrc r = adam_rsrc(p);
#pragma unroll
    for (int f = 0; f < MF - HAND; ++f)
      adam_tile(p, r, acc[f / TN][f % TN], m0 + wm * WM + (f / TN) * 32, n0 + wn * WN + (f % TN) * 32 + (lane & 31), lane >> 5);
  } else {
    epilogue<TM, TN, EPI, TM_LDW_VB>(p, acc, m0 + wm * WM, n0 + wn * WN, lane & 31, lane >> 5);
  }
}

// =================================================================================================
// alternating kernel: eight waves, the two waves of every SIMD take turns at the matrix core
// =================================================================================================
// A block of eight waves puts two waves on each SIMD (waves w and w + 4).  Time is cut into slots; in a slot
// the waves of one half run nothing but the MFMAs of one whole 64-element step, operands already in
// registers, while the waves of the other half fetch THEIR operands of a step from LDS; at the slot's end
// (one barrier) the halves swap.  The matrix core of a SIMD is fed by one wave at a time with no waits inside
// the run, and all LDS and global traffic of the other wave hides behind it.
//   slot 2k:    first half computes step k;        second half reads its fragments of step k
//   slot 2k+1:  first half reads step k+1;         second half computes step k
// Stage k&1 of LDS is free once the second half has read step k (end of slot 2k): every wave then issues its
// share of the global loads of step k+2 into it (start of slot 2k+1) and waits for them before the barrier
// that ends slot 2k+2, two slots later.  A fragment set of a whole step lives in registers (96 of them for a
// 128x64 wave tile) beside the 128 accumulators.
template <int BM, int BN, int BK, int WGM, int WGN, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(512, 1) void gemm_alt_kernel(const MfmaGemmParams p) {
  static_assert(WGM * WGN == 8, "two waves per SIMD");
  extern __shared__ __align__(16) char lds[];
  constexpr int NW = 8;
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
  typedef typename DirectSel<BM, BK, A_KC, NW>::type LA;
  typedef typename DirectSel<BN, BK, B_KC, NW>::type LB;
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  constexpr int LOADS = LA::NLOAD + LB::NLOAD;
  constexpr int KS = BK / 16;

  int m0, n0;
  tile_of_block(p, BM, BN, m0, n0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const bool second = wave >= 4;  // waves w and w + 4 share a SIMD

  LA la;
  LB lb;
  const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
  la.init(p.lda, m0, wave, lane);
  lb.init(p.ldb, n0, wave, lane);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (p.K + BK - 1) / BK;
  bf16x8 fa[KS][TM], fb[KS][TN];
  // this wave's share of the loads of step `step` (never past K: a surplus fetch repeats the last step)
  auto issue = [&](int step) {
    const int k0 = (step < nk ? step : nk - 1) * BK;
    char *st = lds + (step & 1) * STAGE;
    la.issue(ra, st, k0, p.lda, wave);
    lb.issue(rb, st + LA::BYTES, k0, p.ldb, wave);
  };
  // Fragment addresses of an operand with contiguous reduction axis: row r of the tile, 16-byte chunk
  // (2 ks + lane/32) ^ swz(r).  swz looks at row bits 0..5 only and 32 rows further on it flips bit 2, so
  // eight per-lane offsets (slice ks, row-block parity) serve every 32-row block through the instruction's
  // immediate offset; without this the compiler keeps one address register per (block, slice).
  uint32_t ka[KS][2], kb[KS][2];
  {
    const int l32 = lane & 31, hh = lane >> 5;
    const int sw = (l32 ^ (l32 >> 3)) & 7;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const uint32_t o = (uint32_t)(l32 * LA::ROWB + ((((2 * ks + hh) ^ sw ^ (4 * par)) & 7) << 4));
        ka[ks][par] = o + (uint32_t)(wm * WM * (A_KC ? LA::ROWB : 0));
        kb[ks][par] = o + (uint32_t)(wn * WN * (B_KC ? LB::ROWB : 0)) + (uint32_t)LA::BYTES;
      }
  }
  auto read_frags = [&](int step) {
    const char *as = lds + (step & 1) * STAGE, *bs = as + LA::BYTES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if constexpr (A_KC) fa[ks][i] = *reinterpret_cast<const bf16x8 *>(as + ka[ks][i & 1] + i * 32 * LA::ROWB);
        else fa[ks][i] = LA::frag(as, wm * WM + i * 32, ks, lane);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (B_KC) fb[ks][j] = *reinterpret_cast<const bf16x8 *>(as + kb[ks][j & 1] + j * 32 * LB::ROWB);
        else fb[ks][j] = LB::frag(bs, wn * WN + j * 32, ks, lane);
      }
    }
  };
  auto compute = [&]() {
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma_for<EPI>(fa[ks][i], fb[ks][j], acc[i][j]);
    __builtin_amdgcn_s_setprio(0);
  };
  auto slot_end = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };

  issue(0);
  issue(1);
  wait_vmcnt<LOADS>();  // this wave's loads of step 0 have landed (loads complete in order)
  slot_end();
  if (!second) {
    read_frags(0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    slot_end();
    for (int k = 0; k < nk; ++k) {
      compute();                                                   // slot 2k
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // own loads of step k+1
      slot_end();
      issue(k + 2);                                                // slot 2k+1: stage k&1 is free
      if (k + 1 < nk) read_frags(k + 1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      slot_end();
    }
  } else {
    slot_end();
    for (int k = 0; k < nk; ++k) {
      read_frags(k);                                               // slot 2k
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // fragments here; own loads of step k+1 landed
      slot_end();
      issue(k + 2);                                                // slot 2k+1
      compute();
      slot_end();
    }
  }
  wait_vmcnt<0>();  // drain the look-ahead loads before the block may exit
  if constexpr (EPI == 0) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();  // every wave's loads have landed and its LDS reads are done: the stages are free
    epilogue_lds<BM, BN, NW, TM, TN>(p, acc, lds, m0, n0, wm * WM, wn * WN, lane);
  } else {
    epilogue<TM, TN, EPI>(p, acc, m0 + wm * WM, n0 + wn * WN, lane & 31, lane >> 5);
  }
}

// =================================================================================================
// staged kernel (any K that is a multiple of 8): 128x128x64, registers in between
// =================================================================================================
constexpr int SBK = 64, SROWB = SBK * 2;
__device__ __forceinline__ int sswz(int row) { return (row ^ (row >> 3)) & 7; }

template <int R> struct StagedKC {
  static constexpr int NCH = R / 32;
  u32x4 reg[NCH];
  uint32_t voff[NCH];
  __device__ __forceinline__ void init(int64_t ld, int row0) {
    const int c = threadIdx.x & 7, r0 = threadIdx.x >> 3;
#pragma unroll
    for (int i = 0; i < NCH; ++i) voff[i] = (uint32_t)(((int64_t)(row0 + r0 + 32 * i) * ld + c * 8) * 2);
  }
  __device__ __forceinline__ void g2r(rsrc_t rs, int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) reg[i] = buf_load16(rs, voff[i], (uint32_t)k0 * 2);
  }
  // the mask is applied here, after the MFMAs that overlap the loads, so that it forces no early wait
  __device__ __forceinline__ void r2s(char *lds, int k_left) const {
    const int c = threadIdx.x & 7, r0 = threadIdx.x >> 3;
    const bool drop = c * 8 >= k_left;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int r = r0 + 32 * i;
      u32x4 v = reg[i];
      if (drop) v = u32x4{0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4 *>(lds + r * SROWB + ((c ^ sswz(r)) << 4)) = v;
    }
  }
};

template <int R> struct StagedKS {
  static constexpr int RB = R / 8, KG_STEP = 256 / RB, NB = 16 / KG_STEP;
  u32x4 reg[NB][4];
  uint32_t voff[NB];
  int64_t ldb2;
  __device__ __forceinline__ void init(int64_t ld, int row0) {
    const int rb = threadIdx.x % RB, kg0 = threadIdx.x / RB;
    ldb2 = ld * 2;
#pragma unroll
    for (int i = 0; i < NB; ++i) voff[i] = (uint32_t)(((int64_t)(kg0 + i * KG_STEP) * 4 * ld + row0 + rb * 8) * 2);
  }
  __device__ __forceinline__ void g2r(rsrc_t rs, int k0) {
    const uint32_t base = (uint32_t)((int64_t)k0 * ldb2);
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) reg[i][j] = buf_load16(rs, voff[i] + (uint32_t)(j * ldb2), base);
  }
  // 4 k-rows x 8 columns per thread are transposed in registers into 8 pieces of 4 k-values
  __device__ __forceinline__ void r2s(char *lds, int /*k_left*/) const {
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
        *reinterpret_cast<u32x2 *>(lds + r * SROWB + (((kg >> 1) ^ sswz(r)) << 4) + ((kg & 1) << 3)) = o;
      }
    }
  }
};
template <int R, bool KC> struct StagedSel { typedef StagedKC<R> type; };
template <int R> struct StagedSel<R, false> { typedef StagedKS<R> type; };

template <bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256) void gemm_staged_kernel(const MfmaGemmParams p) {
  constexpr int BM = 128, BN = 128, WM = 64, WN = 64, TM = 2, TN = 2;
  constexpr int A_BYTES = BM * SROWB, STAGE = (BM + BN) * SROWB;
  __shared__ __align__(16) char lds[2 * STAGE];
  int m0, n0;
  tile_of_block(p, BM, BN, m0, n0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, hh = lane >> 5;
  typename StagedSel<BM, A_KC>::type la;
  typename StagedSel<BN, B_KC>::type lb;
  const rsrc_t ra = make_rsrc(p.A, p.a_bytes), rb = make_rsrc(p.B, p.b_bytes);
  la.init(p.lda, m0);
  lb.init(p.ldb, n0);
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int nk = (p.K + SBK - 1) / SBK;
  la.g2r(ra, 0);
  lb.g2r(rb, 0);
  la.r2s(lds, p.K);
  lb.r2s(lds + A_BYTES, p.K);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.g2r(ra, (kt + 1) * SBK);
      lb.g2r(rb, (kt + 1) * SBK);
    }
    const char *As = lds + cur * STAGE, *Bs = As + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < SBK / 16; ++ks) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = wm * WM + i * 32 + l32;
        a[i] = *reinterpret_cast<const bf16x8 *>(As + r * SROWB + (((2 * ks + hh) ^ sswz(r)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = wn * WN + j * 32 + l32;
        b[j] = *reinterpret_cast<const bf16x8 *>(Bs + r * SROWB + (((2 * ks + hh) ^ sswz(r)) << 4));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma_for<EPI>(a[i], b[j], acc[i][j]);
    }
    if (kt + 1 < nk) {
      char *nx = lds + (cur ^ 1) * STAGE;
      la.r2s(nx, p.K - (kt + 1) * SBK);
      lb.r2s(nx + A_BYTES, p.K - (kt + 1) * SBK);
    }
    __syncthreads();
  }
  epilogue<TM, TN, EPI>(p, acc, m0 + wm * WM, n0 + wn * WN, l32, hh);
}

// =================================================================================================
// host side: one layout (A_KC, B_KC, EPI) per translation unit, so that the variants compile in parallel
// =================================================================================================
template <bool A_KC, bool B_KC, int EPI> static MfmaGemmParams make_params(const GemmArgs &g, int BM, int BN) {
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
  p.a_bytes = (uint32_t)((A_KC ? g.M * g.a_rs : g.K * g.a_cs) * 2);
  p.b_bytes = (uint32_t)((B_KC ? g.N * g.b_rs : g.K * g.b_cs) * 2);
  p.c_bytes = (uint32_t)(g.M * g.ldc * (EPI == 0 ? 2 : 4));
  if (EPI == 3 && g.adam) p.adam = *g.adam;
  p.stagger_ticks = p.stagger_phases = p.stagger_blocks = 0;
  return p;
}
// Start offsets for a fused-update product on one large block per compute unit (see stagger_by_unit): two groups of
// units, the second one main loop late (a 256x192 tile at about 4.5 TFLOP/s a unit).  TM_GEMM_STAGGER_US overrides the
// span (twice the delay of the second group; 0 switches the offsets off), TM_GEMM_STAGGER_PHASES the number of groups.
static void stagger_of(MfmaGemmParams &p, int BM, int BN, int64_t nblk) {
  static int cus = 0, khz = 0, phases = 2;
  static double forced = -1.0;
  if (!cus) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || cus <= 0 || khz <= 0)
      cus = -1;
    if (const char *e = getenv("TM_GEMM_STAGGER_US")) forced = atof(e);
    if (const char *e = getenv("TM_GEMM_STAGGER_PHASES")) phases = atoi(e) > 1 ? atoi(e) : 2;
  }
  if (cus <= 0 || nblk < 2 * (int64_t)cus) return;
  const double main_loop_us = 2.0 * BM * BN * (double)p.K / 4.5e6;
  const double us = forced >= 0.0 ? forced : 2.0 * main_loop_us;
  if (us <= 0.0) return;
  p.stagger_ticks = (int)(us * khz * 1e-3);
  p.stagger_phases = phases;
  p.stagger_blocks = cus;
}

static std::string kernel_tag(const char *base, int bm, int bn, int wgm, int wgn, bool akc, bool bkc, int epi) {
  return std::string(base) + "<" + std::to_string(bm) + "x" + std::to_string(bn) + ",waves " + std::to_string(wgm) + "x" +
         std::to_string(wgn) + "," + (akc ? "kc" : "ks") + "," + (bkc ? "kc" : "ks") + ",epi" + std::to_string(epi) + ">";
}

template <int BM, int BN, int WGM, int WGN, bool A_KC, bool B_KC, int EPI, int NSA = 2, int NSB = 2>
static int launch_pipe(const GemmArgs &g, hipStream_t s) {
  constexpr int BK = GEMM_BK;
  const MfmaGemmParams p = make_params<A_KC, B_KC, EPI>(g, BM, BN);
  constexpr int lds_bytes = (NSA * BM + NSB * BN) * BK * 2 > BM * BN * 2 ? (NSA * BM + NSB * BN) * BK * 2 : BM * BN * 2;
  static_assert(lds_bytes <= 160 * 1024, "LDS");
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_pipe_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, EPI, NSA, NSB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
      return fail(TM_ELAUNCH, "gemm_mfma: cannot reserve %d bytes of LDS", lds_bytes);
    attr_set = true;
  }
  const int64_t nblk = (int64_t)p.tiles_m * p.tiles_n;
  if (nblk > 0x7fffffff) return fail(TM_ESIZE, "gemm_mfma: too many tiles");
  static const std::string name = kernel_tag(NSB == 3 ? (NSA == 3 ? "gemm_pipe33_kernel" : "gemm_pipe23_kernel") : "gemm_pipe_kernel", BM, BN, WGM, WGN, A_KC, B_KC, EPI);
  g_last_kernel = name.c_str();
  if (EPI == 3 && !g.adam) return fail(TM_EINVAL, "gemm_mfma: the fused update needs its target");
  if (g.k_splits > 1 && (EPI != 2 || g.K % ((int64_t)BK * g.k_splits) != 0))
    return fail(TM_EINVAL, "gemm_mfma: split reduction needs whole steps per part and fp32 results");
  gemm_pipe_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, EPI, NSA, NSB>
      <<<dim3((unsigned)nblk, (unsigned)(g.k_splits > 1 ? g.k_splits : 1)), 64 * WGM * WGN, lds_bytes, s>>>(p);
  return check_launch("gemm_pipe");
}

template <int BM, int BN, int WGM, int WGN, bool A_KC, bool B_KC, int EPI>
static int launch_alt(const GemmArgs &g, hipStream_t s) {
  constexpr int BK = GEMM_BK;
  const MfmaGemmParams p = make_params<A_KC, B_KC, EPI>(g, BM, BN);
  constexpr int lds_bytes = 2 * (BM + BN) * BK * 2;
  static_assert(lds_bytes <= 160 * 1024, "LDS");
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_alt_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, EPI>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
      return fail(TM_ELAUNCH, "gemm_mfma: cannot reserve %d bytes of LDS", lds_bytes);
    attr_set = true;
  }
  const int64_t nblk = (int64_t)p.tiles_m * p.tiles_n;
  if (nblk > 0x7fffffff) return fail(TM_ESIZE, "gemm_mfma: too many tiles");
  if (g.k_splits > 1) return fail(TM_EINVAL, "gemm_mfma: the alternating kernel does not split the reduction");
  static const std::string name = kernel_tag("gemm_alt_kernel", BM, BN, WGM, WGN, A_KC, B_KC, EPI);
  g_last_kernel = name.c_str();
  gemm_alt_kernel<BM, BN, BK, WGM, WGN, A_KC, B_KC, EPI><<<dim3((unsigned)nblk), 512, lds_bytes, s>>>(p);
  return check_launch("gemm_alt");
}

template <int BM, int BN, int WGM, int WGN, int NP, bool A_KC, bool B_KC, int EPI>
static int launch_ldw(const GemmArgs &g, hipStream_t s) {
  constexpr int BK = GEMM_BK;
  MfmaGemmParams p = make_params<A_KC, B_KC, EPI>(g, BM, BN);
  if (EPI == 3 && NP == 4) stagger_of(p, BM, BN, (int64_t)p.tiles_m * p.tiles_n);
  constexpr int lds_bytes = 2 * (BM + BN) * BK * 2 > BM * BN * 2 ? 2 * (BM + BN) * BK * 2 : BM * BN * 2;
  static_assert(lds_bytes <= 160 * 1024, "LDS");
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_ldw_kernel<BM, BN, BK, WGM, WGN, NP, A_KC, B_KC, EPI>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
      return fail(TM_ELAUNCH, "gemm_mfma: cannot reserve %d bytes of LDS", lds_bytes);
    attr_set = true;
  }
  const int64_t nblk = (int64_t)p.tiles_m * p.tiles_n;
  if (nblk > 0x7fffffff) return fail(TM_ESIZE, "gemm_mfma: too many tiles");
  if (g.k_splits > 1 && (EPI != 2 || g.K % ((int64_t)BK * g.k_splits) != 0))
    return fail(TM_EINVAL, "gemm_mfma: split reduction needs whole steps per part and fp32 results");
  if (EPI == 3 && !g.adam) return fail(TM_EINVAL, "gemm_mfma: the fused update needs its target");
  static const std::string name = kernel_tag(NP == 4 ? "gemm_ldw4_kernel" : "gemm_ldw2_kernel", BM, BN, WGM, WGN, A_KC, B_KC, EPI);
  g_last_kernel = name.c_str();
  gemm_ldw_kernel<BM, BN, BK, WGM, WGN, NP, A_KC, B_KC, EPI>
      <<<dim3((unsigned)nblk, (unsigned)(g.k_splits > 1 ? g.k_splits : 1)), 64 * (WGM * WGN + NP), lds_bytes, s>>>(p);
  return check_launch("gemm_ldw");
}

template <bool A_KC, bool B_KC, int EPI> static int launch_staged(const GemmArgs &g, hipStream_t s) {
  const MfmaGemmParams p = make_params<A_KC, B_KC, EPI>(g, 128, 128);
  static const std::string name = kernel_tag("gemm_staged_kernel", 128, 128, 2, 2, A_KC, B_KC, EPI);
  g_last_kernel = name.c_str();
  gemm_staged_kernel<A_KC, B_KC, EPI><<<dim3((unsigned)(p.tiles_m * p.tiles_n)), 256, 0, s>>>(p);
  return check_launch("gemm_staged");
}

// The tile configurations (BM, BN, wave grid).  gemm_mfma.hip holds the same list with each entry's
// occupancy and measured relative speed, in the same order.
// configurations of the alternating kernel follow those of the pipelined one in the numbering
#define TM_GEMM_ALT_CONFIGS(X) X(256, 256, 2, 4) X(256, 256, 4, 2)
// ... then the pipelined kernel with three LDS stages of both tiles (tiles whose three stages fit 160 KB)
#define TM_GEMM_PIPE33_CONFIGS(X) X(256, 128, 4, 2) X(128, 256, 2, 4)
// ... then the kernel with loader waves (eight multiplying waves and four loaders)
#define TM_GEMM_LDW_CONFIGS(X) X(256, 192, 4, 2, 4) X(128, 192, 2, 2, 2) X(256, 192, 4, 2, 2)
#define TM_GEMM_CONFIGS(X) \
  X(128, 192, 2, 2) X(128, 128, 2, 2) X(192, 128, 2, 2) X(256, 192, 4, 2) X(192, 256, 2, 4) X(256, 256, 2, 4) \
  X(256, 256, 4, 2) X(256, 128, 4, 2) X(256, 192, 2, 2)

// The variants the host side launches are instantiated explicitly (an implicit instantiation from inside
// the launcher templates leaves the host-side kernel handle undefined with this compiler).
#define TM_GEMM_INSTANTIATE_ONE(BM_, BN_, WGM_, WGN_, AKC, BKC, EPI) \
  template __global__ void gemm_pipe_kernel<BM_, BN_, GEMM_BK, WGM_, WGN_, AKC, BKC, EPI>(const MfmaGemmParams);
#define TM_GEMM_INSTANTIATE(AKC, BKC, EPI)                  \
  TM_GEMM_INSTANTIATE_ONE(128, 192, 2, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(128, 128, 2, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(192, 128, 2, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(256, 192, 4, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(192, 256, 2, 4, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(256, 256, 2, 4, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(256, 256, 4, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(256, 128, 4, 2, AKC, BKC, EPI)    \
  TM_GEMM_INSTANTIATE_ONE(256, 192, 2, 2, AKC, BKC, EPI)    \
  template __global__ void gemm_alt_kernel<256, 256, GEMM_BK, 2, 4, AKC, BKC, EPI>(const MfmaGemmParams); \
  template __global__ void gemm_alt_kernel<256, 256, GEMM_BK, 4, 2, AKC, BKC, EPI>(const MfmaGemmParams); \
  template __global__ void gemm_pipe_kernel<256, 128, GEMM_BK, 4, 2, AKC, BKC, EPI, 3, 3>(const MfmaGemmParams); \
  template __global__ void gemm_pipe_kernel<128, 256, GEMM_BK, 2, 4, AKC, BKC, EPI, 3, 3>(const MfmaGemmParams); \
  template __global__ void gemm_ldw_kernel<256, 192, GEMM_BK, 4, 2, 4, AKC, BKC, EPI>(const MfmaGemmParams); \
  template __global__ void gemm_ldw_kernel<128, 192, GEMM_BK, 2, 2, 2, AKC, BKC, EPI>(const MfmaGemmParams); \
  template __global__ void gemm_ldw_kernel<256, 192, GEMM_BK, 4, 2, 2, AKC, BKC, EPI>(const MfmaGemmParams);

// config: index into the list above, as chosen by gemm_mfma_config()
template <bool A_KC, bool B_KC, int EPI> static int launch_layout(const GemmArgs &g, int config, hipStream_t s) {
  if (g.K % GEMM_BK != 0) return launch_staged<A_KC, B_KC, EPI>(g, s);  // the pipelined kernel takes whole steps only
  int idx = 0;
#define X(BM_, BN_, WGM_, WGN_) \
  if (config == idx++) return launch_pipe<BM_, BN_, WGM_, WGN_, A_KC, B_KC, EPI>(g, s);
  TM_GEMM_CONFIGS(X)
#undef X
#define X(BM_, BN_, WGM_, WGN_) \
  if (config == idx++) return launch_alt<BM_, BN_, WGM_, WGN_, A_KC, B_KC, EPI>(g, s);
  TM_GEMM_ALT_CONFIGS(X)
#undef X
#define X(BM_, BN_, WGM_, WGN_) \
  if (config == idx++) return launch_pipe<BM_, BN_, WGM_, WGN_, A_KC, B_KC, EPI, 3, 3>(g, s);
  TM_GEMM_PIPE33_CONFIGS(X)
#undef X
#define X(BM_, BN_, WGM_, WGN_, NP_) \
  if (config == idx++) return launch_ldw<BM_, BN_, WGM_, WGN_, NP_, A_KC, B_KC, EPI>(g, s);
  TM_GEMM_LDW_CONFIGS(X)
#undef X
  return fail(TM_EINVAL, "gemm_mfma: no tile configuration %d", config);
}

}  // namespace tmk

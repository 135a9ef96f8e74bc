// Flash-style causal grouped-query attention for gfx950, head_dim 128, bf16 storage, fp32 softmax and
// accumulation, v_mfma_f32_32x32x16_bf16 throughout.  Three kernels: forward, dQ, and dK/dV.  The
// [S,S] score matrix never exists; only the per-row log-sum-exp is kept for the backward pass.
//
// Orientation.  An MFMA 32x32 result leaves each lane with ONE column (lane % 32) and 16 of the 32 rows.
// Every product is therefore arranged so that the index a lane needs a scalar for is the column:
//   forward / dQ : S^T = K Q^T (rows = keys, columns = queries) -> the running max / sum, lse and delta
//                  of a query are per-lane scalars, and a row reduction is 16 in-lane steps plus one
//                  exchange with lane ^ 32;
//   dK/dV        : S = Q K^T (rows = queries, columns = keys)   -> the dK/dV columns of a key stay in
//                  one lane.
// In both cases the probabilities come out of the MFMA exactly in the register layout that the next
// MFMA wants for its B operand (8 contraction values per lane), provided the A operand enumerates the
// contraction index in the same order {4g..4g+3, 8+4g..8+4g+3} (g = lane / 32).  That A operand (V^T,
// K^T, dO^T, Q^T) is read from the row-major LDS tile with the transposing LDS read
// ds_read_b64_tr_b16, so nothing is ever transposed through registers or HBM.
//
// Tiles.  Forward and dQ: one block = 128 queries of one head (4 waves x 32 queries, Q in registers; capped
// at 256 VGPRs so that two blocks share a CU and one block's softmax overlaps the other's MFMAs),
// K/V streamed in 64-key tiles, double buffered in LDS.  dK/dV: one block = 128 keys of one kv
// head (4 waves x 32 keys, K [and V] in registers), Q/dO streamed in tiles of 32 (dV pass) or 64 (dK pass)
// queries for each of the G query heads of the group, so dK/dV are summed over the group in registers: no
// atomics, deterministic.  dV and dK are two launches of one template: a fused pass needs 350 registers (K, V
// fragments and two 32x128 accumulators), i.e. one block per CU with nothing to hide the exponentials behind;
// the two halves need 168 and 212, run 3 and 2 blocks per CU, and together take 0.7x the fused time although
// S = Q K^T is computed twice.
// Every streamed tile reaches LDS by LDS-DMA loads (no staging registers); operand fragments are read from LDS
// through small register rings, a few MFMAs ahead of their use.
// Causality: tiles entirely above the diagonal are never loaded; heavy blocks are scheduled first; the
// per-element causal test is made only by the (wave-uniformly chosen) tiles that touch the diagonal.
#include <type_traits>

#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

namespace {

constexpr int D = 128;          // head_dim
constexpr int PITCH = D + 8;    // LDS row pitch in elements (272 B = 4 banks past a multiple of 64)
// Streamed tiles (K, V, Q, dO) keep row r of the tile in LDS row perm(r): inside every group of 16 rows the two
// 2-bit fields of the row number are exchanged.  A row read (16 lanes = 16 consecutive tile rows, 16 bytes each)
// still meets 16 different LDS rows, 4 banks apart: all 64 banks once.  A transposing read (32 lanes = 4
// consecutive tile rows x 64 contiguous bytes) now meets LDS rows that are 4 apart, i.e. 16 banks apart: four
// disjoint windows.  With the rows in natural order those four windows overlapped (4 banks apart), and half of all
// LDS cycles of the three kernels were bank-conflict cycles (by counter).  Every address stays base + constant.
__device__ __forceinline__ int perm(int r) { return (r & ~15) | ((r & 3) << 2) | ((r >> 2) & 3); }
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ f32x16_t mfma(u32x4_t a, u32x4_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// A/B operand whose contraction index is contiguous in the LDS tile: tile row row0 + r with row0 a multiple of 16
// and prow = perm(r) (computed once per lane)
__device__ __forceinline__ u32x4_t frag(const bf16_t* tile, int row0, int prow, int kofs) {
  return *reinterpret_cast<const u32x4_t*>(tile + (row0 + prow) * PITCH + kofs);
}

// A operand taken from the tile TRANSPOSED: tile is [k][PITCH] (k = contraction index, 16 rows starting
// at kbase), the operand row is the tile column nbase + lane % 32, and the 8 contraction values of the
// lane are k = kbase + {4g..4g+3, 8+4g..8+4g+3}.
__device__ __forceinline__ u32x4_t frag_tr(const bf16_t* tile, int kbase, int nbase, int lane) {
  const int g = lane >> 5;
  const int l16 = lane & 15;
  const int col = nbase + ((lane >> 4) & 1) * 16 + (l16 & 3) * 4;
  const int row = kbase + ((l16 >> 2) << 2) + g;   // perm(kbase + 4 g + (l16 >> 2)); kbase is a multiple of 16
  typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
  const bf16_t* p0 = tile + row * PITCH + col;
  const bf16_t* p1 = p0 + 2 * PITCH;                // perm of the tile row 8 further on
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p1));
  u32x2_t a = __builtin_bit_cast(u32x2_t, lo), b = __builtin_bit_cast(u32x2_t, hi);
  u32x4_t r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  return r;
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return f2bf2(lo, hi);
}

// registers q0..q0+7 of a 32x32 accumulator -> the 8-value B operand of the next MFMA
__device__ __forceinline__ u32x4_t pack_half(const f32x16_t& v, int half) {
  u32x4_t r;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    r[w] = pack2(v[half * 8 + 2 * w], v[half * 8 + 2 * w + 1]);
  return r;
}

// row index (0..31) that accumulator register q of this lane holds
__device__ __forceinline__ int acc_row(int q, int g) { return 8 * (q >> 2) + 4 * g + (q & 3); }

// Staging of a tile of 64 or 32 rows x 128 columns (bf16) of a row-major global matrix in LDS, without registers:
// LDS-DMA loads (16 bytes per lane straight into LDS, written as instructions so that the waits are this file's
// own: the compiler does not see that they write LDS).  A 64-row tile with its 272-byte
// pitch is 17 chunks of 1 KiB of consecutive LDS bytes; wave w issues the chunks w, w + 4, ... and lane l of chunk c
// fills the bytes c * 1024 + 16 l .. + 16, i.e. LDS row (c * 1024 + 16 l) / 272 = tile row perm(LDS row), 16-byte
// piece ((c * 1024 + 16 l) % 272) / 16; the 17th piece of a row is its padding and loads from beyond the buffer
// (zeros).  Rows past the end of the sequence lie beyond the buffer as well.
__device__ __forceinline__ i32x4_t rsrc_words(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)base;
  i32x4_t r;
  r[0] = (int)(uint32_t)a; r[1] = (int)((uint32_t)(a >> 32) & 0xffffu); r[2] = (int)bytes; r[3] = 0x00020000;
  return r;
}
__device__ __forceinline__ void dma16(i32x4_t rs, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rs) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const bf16_t* p) {
  typedef __attribute__((address_space(3))) const bf16_t* lds_p;
  return (uint32_t)(uintptr_t)(lds_p)p;
}
template <int ROWS>   // rows of the tile (64, or 32: 8.5 chunks, the second half of the ninth is not part of the tile)
struct TileDma {
  static constexpr int BYTES = ROWS * PITCH * 2;
  static constexpr int CHUNKS = (BYTES + 1023) / 1024;   // 17 / 9
  static constexpr int PER_WAVE = (CHUNKS + 3) / 4;      // 5 / 3 (the last only in wave 0)
  uint32_t voff[PER_WAVE];   // byte offset of the lane's piece from the tile's first element (beyond any buffer: padding)
  __device__ __forceinline__ void init(int ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int o = (wave + 4 * i) * 1024 + lane * 16;
      const int R = o / (PITCH * 2), piece = (o % (PITCH * 2)) / 16;
      // 2^31 plus any offset inside a sequence (below 2^31, see attn_mfma_supported) stays beyond the buffer and does not wrap
      voff[i] = (piece < 16 && o < BYTES) ? (uint32_t)(perm(R) * ld + piece * 8) * 2u : 0x80000000u;
    }
  }
  // tile_bytes: byte offset of the tile's first element in the buffer; wave_s: the wave index as a scalar
  __device__ __forceinline__ void issue(i32x4_t rs, const bf16_t* tile, uint32_t tile_bytes, int wave_s) const {
    const uint32_t base = lds_address(tile);
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i)
      if (wave_s + 4 * i < CHUNKS) dma16(rs, base + (uint32_t)(wave_s + 4 * i) * 1024u, voff[i] + tile_bytes);
  }
};
#define TIDE_ATTN_WAIT_DMA() __builtin_amdgcn_s_waitcnt(0x0F70)   /* vmcnt(0) */

// Write a wave's 32 x 128 result, held transposed in 4 accumulators (acc[ct] = rows ct*32.., column =
// lane % 32 = the wave-local output row), into an LDS tile [128][PITCH] at rows wave*32.. as bf16.
__device__ __forceinline__ void stage_out(bf16_t* tile, const f32x16_t (&acc)[4], float mul, int wave, int lane) {
  const int g = lane >> 5, r = wave * 32 + (lane & 31);
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int qq = 0; qq < 4; ++qq) {
      const int c = ct * 32 + 8 * qq + 4 * g;
      uint2 v;
      v.x = pack2(acc[ct][qq * 4 + 0] * mul, acc[ct][qq * 4 + 1] * mul);
      v.y = pack2(acc[ct][qq * 4 + 2] * mul, acc[ct][qq * 4 + 3] * mul);
      *reinterpret_cast<uint2*>(tile + r * PITCH + c) = v;
    }
}

// Copy the staged [128][128] tile to global rows row0.. (< row_end) of a matrix with leading dim ld.
__device__ __forceinline__ void copy_out(const bf16_t* tile, bf16_t* dst, int64_t row0, int64_t row_end, int ld,
                                         int col0, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int p = tid + i * 256;
    const int row = p >> 4, piece = p & 15;
    if (row0 + row < row_end)
      *reinterpret_cast<i32x4_t*>(dst + (size_t)(row0 + row) * ld + col0 + piece * 8) =
          *reinterpret_cast<const i32x4_t*>(tile + row * PITCH + piece * 8);
  }
}

constexpr int BQ = 128, BKV = 64;
constexpr int KV_TILE = BKV * PITCH;  // elements

// Depth of the operand-fragment rings of the three kernels (0 in the dQ kernel: the plain loop).  Measured when the tiles
// were still staged through registers, backward at 16 x 2048 / 2 x 16384: dQ 0 / dK-dV 4: 3.56 / 21.4 ms; 2 / 4: 3.48 /
// 21.0; 4 / 4: 3.79 / 22.7 (the dQ kernel, then at 256 registers, spilled with a ring of four); 0 / 2: 3.60 / 21.2;
// before the rings 3.65 / 21.6.  With LDS-DMA tile loads (dQ at 233 registers) depths of 2 to 6 measure the same.
#ifndef TIDE_ATTN_DQ_RING
#define TIDE_ATTN_DQ_RING 2
#endif
#ifndef TIDE_ATTN_DKV_RING
#define TIDE_ATTN_DKV_RING 4
#endif
#ifndef TIDE_ATTN_KRING
#define TIDE_ATTN_KRING 4
#endif
// Work item (x, y, z) of an nx * ny * nz problem from the block's place in the 1-D dispatch order.
// Work-groups go to the 8 XCDs round-robin and every XCD has its own L2.  The blocks of a "group" (all x of gy
// consecutive y of one z: the query blocks of the heads that share a kv head, or the key blocks of one kv
// head) stream the same K/V resp. Q/dO rows, so a whole group is given to ONE XCD, group after group, x
// fastest.  With the plain (x, y, z) order the 16 key blocks of a kv head were spread over all XCDs and the
// dK / dV passes hit L2 on 2 % of their requests.  Falls back to the plain order when the number of
// groups is not a multiple of 8.
struct Work3 { int x, y, z; };
__device__ __forceinline__ Work3 xcd_group_work(int nx, int ny, int nz, int gy) {
  const int n = blockIdx.x;
  const int per_group = nx * gy, groups_per_z = ny / gy, ngroups = groups_per_z * nz;
  int grp, in_g;
  if ((ngroups & 7) == 0) {
    const int xcd = n & 7, slot = n >> 3;
    grp = (slot / per_group) * 8 + xcd;
    in_g = slot % per_group;
  } else {
    grp = n / per_group;
    in_g = n % per_group;
  }
  Work3 w;
  w.x = in_g % nx;
  w.y = (grp % groups_per_z) * gy + in_g / nx;
  w.z = grp / groups_per_z;
  return w;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                            float* __restrict__ lse, int Smax, int nh, int nkv,
                                                            const int* __restrict__ cu, int64_t T, int nseq) {
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sK = smem;                 // [2][KV_TILE]
  bf16_t* sV = smem + 2 * KV_TILE;   // [2][KV_TILE]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5, plr = perm(lr);
  const int nqb = (Smax + BQ - 1) / BQ;
  const Work3 wk = xcd_group_work(nqb, nh, nseq, nh / nkv);
  const int qb = nqb - 1 - wk.x;  // heavy (late) query blocks first
  const int h = wk.y, b = wk.z;
  const SeqView sv = seq_view(cu, b, Smax, T);
  const int S = sv.len;
  const int G = nh / nkv, kh = h / G;
  const int ld = (nh + 2 * nkv) * D;
  const int q0 = qb * BQ, qw = q0 + wave * 32, iq = qw + lr;
  if (q0 >= S) return;   // the whole block, before any barrier: this sequence is shorter
  const bf16_t* base = qkv + (size_t)sv.row0 * ld;
  const __amdgpu_buffer_rsrc_t rs = rsrc(base, (uint32_t)((size_t)S * ld * 2));
  const int kcol = (nh + kh) * D, vcol = (nh + nkv + kh) * D;
  const float c = kLog2e / sqrtf((float)D);

  u32x4_t qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    qf[kk] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, ((uint32_t)iq * (uint32_t)ld + (uint32_t)(h * D + kk * 16 + g * 8)) * 2u, 0, 0));

  f32x16_t o[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int q = 0; q < 16; ++q) o[ct][q] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int kv_end = min(S, q0 + BQ);
  const int nt = (kv_end + BKV - 1) / BKV;
  const i32x4_t rsw = rsrc_words(base, (uint32_t)((size_t)S * ld * 2));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  TileDma<64> dma;
  dma.init(ld, wave, lane);
  dma.issue(rsw, sK, (uint32_t)kcol * 2u, wave_s);
  dma.issue(rsw, sV, (uint32_t)vcol * 2u, wave_s);
  // vmcnt(0): nothing of the prologue is in flight inside the loop.  The Q (and dO) fragments are first used there, so
  // the compiler issues their loads last and, at the loop's head, still counts them as outstanding; inside the loop
  // the next tile's eight loads are then younger than they are, and the waits it puts in front of the first MFMAs
  // ("all but 7, 6, ... 0 loads done") make every tile wait for the tile after it to arrive from memory.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int st = t & 1;
    const int j0 = t * BKV;
    if (t + 1 < nt) {   // the next tile, into the stage whose last readers passed the barrier at the end of the step before
      const uint32_t row_bytes = (uint32_t)(j0 + BKV) * (uint32_t)ld * 2u;
      dma.issue(rsw, sK + (st ^ 1) * KV_TILE, row_bytes + (uint32_t)kcol * 2u, wave_s);
      dma.issue(rsw, sV + (st ^ 1) * KV_TILE, row_bytes + (uint32_t)vcol * 2u, wave_s);
    }
    if (j0 <= qw + 31) {  // wave-uniform: the tile has at least one unmasked key for this wave
      const bf16_t* K = sK + st * KV_TILE;
      const bf16_t* V = sV + st * KV_TILE;
      f32x16_t s[2];
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int q = 0; q < 16; ++q) s[jt][q] = 0.f;
      {
        // the 16 K fragments of the tile through a ring of TIDE_ATTN_KRING registers sets: a fragment is requested
        // that many MFMAs before its own (read, wait, MFMA one after the other leaves the LDS latency, three
        // MFMA times, exposed at every step)
        constexpr int RING = TIDE_ATTN_KRING;
        u32x4_t kb[RING];
#pragma unroll
        for (int i = 0; i < RING; ++i) kb[i] = frag(K, (i >> 3) * 32, plr, (i & 7) * 16 + g * 8);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[i >> 3] = mfma(kb[i % RING], qf[i & 7], s[i >> 3]);
          if (i + RING < 16) kb[i % RING] = frag(K, ((i + RING) >> 3) * 32, plr, ((i + RING) & 7) * 16 + g * 8);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (j0 + BKV - 1 > qw) {  // the tile touches the diagonal of this wave
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
          for (int q = 0; q < 16; ++q)
            if (j0 + jt * 32 + acc_row(q, g) > iq) s[jt][q] = -INFINITY;
      }
      float tm = -INFINITY;
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int q = 0; q < 16; ++q) tm = fmaxf(tm, s[jt][q]);
      tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
      const float mn = fmaxf(m, tm);          // finite: key 0 is visible to every query
      const float alpha = __builtin_amdgcn_exp2f((m - mn) * c);
      const float mc = mn * c;
      float ps = 0.f;
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const float p = __builtin_amdgcn_exp2f(s[jt][q] * c - mc);
          s[jt][q] = p;
          ps += p;
        }
      ps += __shfl_xor(ps, 32, 64);
      l = l * alpha + ps;
      m = mn;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // wave-uniform: some row's running max moved
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int q = 0; q < 16; ++q) o[ct][q] *= alpha;
      }
      u32x4_t pf[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) pf[ks] = pack_half(s[ks >> 1], ks & 1);
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) o[ct] = mfma(frag_tr(V, ks * 16, ct * 32, lane), pf[ks], o[ct]);
    }
    TIDE_ATTN_WAIT_DMA();
    __syncthreads();
  }

  const float inv = 1.0f / l;
  stage_out(smem, o, inv, wave, lane);
  if (g == 0 && iq < S) lse[stat_index(cu, T, sv, b, h, nh, Smax, iq)] = m * (1.0f / sqrtf((float)D)) + logf(l);
  __syncthreads();
  copy_out(smem, out, sv.row0 + q0, sv.row0 + min(S, q0 + BQ), nh * D, h * D, tid);
}

// ------------------------------------------------------------------------------------------------
// backward, dQ: same streaming structure as the forward pass
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void attn_dq_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, int Smax, int nh, int nkv,
                                                           const int* __restrict__ cu, int64_t T, int nseq) {
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sK = smem;
  bf16_t* sV = smem + 2 * KV_TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5, plr = perm(lr);
  const int nqb = (Smax + BQ - 1) / BQ;
  const Work3 wk = xcd_group_work(nqb, nh, nseq, nh / nkv);
  const int qb = nqb - 1 - wk.x;
  const int h = wk.y, b = wk.z;
  const SeqView sv = seq_view(cu, b, Smax, T);
  const int S = sv.len;
  const int G = nh / nkv, kh = h / G;
  const int ld = (nh + 2 * nkv) * D, ldo = nh * D;
  const int q0 = qb * BQ, qw = q0 + wave * 32, iq = qw + lr;
  if (q0 >= S) return;   // the whole block, before any barrier
  const __amdgpu_buffer_rsrc_t rs = rsrc(qkv + (size_t)sv.row0 * ld, (uint32_t)((size_t)S * ld * 2));
  const __amdgpu_buffer_rsrc_t rso = rsrc(dout + (size_t)sv.row0 * ldo, (uint32_t)((size_t)S * ldo * 2));
  const int kcol = (nh + kh) * D, vcol = (nh + nkv + kh) * D;
  const float scale = 1.0f / sqrtf((float)D);
  const float c = kLog2e * scale;

  u32x4_t qf[8], dof[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    qf[kk] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, ((uint32_t)iq * (uint32_t)ld + (uint32_t)(h * D + kk * 16 + g * 8)) * 2u, 0, 0));
    dof[kk] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rso, ((uint32_t)iq * (uint32_t)ldo + (uint32_t)(h * D + kk * 16 + g * 8)) * 2u, 0, 0));
  }
  const bool valid = iq < S;
  const bool edge_q = qw + 32 > S;   // wave-uniform: some query row of this wave lies past the sequence
  const float lse_i = valid ? lse[stat_index(cu, T, sv, b, h, nh, Smax, iq)] * kLog2e : 0.f;
  const float del_i = valid ? delta[stat_index(cu, T, sv, b, h, nh, Smax, iq)] : 0.f;

  f32x16_t dq[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int q = 0; q < 16; ++q) dq[ct][q] = 0.f;

  const int kv_end = min(S, q0 + BQ);
  const int nt = (kv_end + BKV - 1) / BKV;
  const i32x4_t rsw = rsrc_words(qkv + (size_t)sv.row0 * ld, (uint32_t)((size_t)S * ld * 2));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  TileDma<64> dma;
  dma.init(ld, wave, lane);
  dma.issue(rsw, sK, (uint32_t)kcol * 2u, wave_s);
  dma.issue(rsw, sV, (uint32_t)vcol * 2u, wave_s);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): nothing of the prologue is in flight inside the loop (see the forward kernel)
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int st = t & 1;
    const int j0 = t * BKV;
    if (t + 1 < nt) {
      const uint32_t row_bytes = (uint32_t)(j0 + BKV) * (uint32_t)ld * 2u;
      dma.issue(rsw, sK + (st ^ 1) * KV_TILE, row_bytes + (uint32_t)kcol * 2u, wave_s);
      dma.issue(rsw, sV + (st ^ 1) * KV_TILE, row_bytes + (uint32_t)vcol * 2u, wave_s);
    }
    if (j0 <= qw + 31) {
      const bf16_t* K = sK + st * KV_TILE;
      const bf16_t* V = sV + st * KV_TILE;
      const bool diag = j0 + BKV - 1 > qw;
      u32x4_t dsf[4];
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        f32x16_t s, dp;
#pragma unroll
        for (int q = 0; q < 16; ++q) { s[q] = 0.f; dp[q] = 0.f; }
#if TIDE_ATTN_DQ_RING == 0
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          s = mfma(frag(K, jt * 32, plr, kk * 16 + g * 8), qf[kk], s);
          dp = mfma(frag(V, jt * 32, plr, kk * 16 + g * 8), dof[kk], dp);
        }
#else
        {
          // K and V fragments alternately through a ring, each requested TIDE_ATTN_DQ_RING MFMAs ahead (see the forward kernel)
          constexpr int RING = TIDE_ATTN_DQ_RING;
          u32x4_t fb[RING];
          auto fetch = [&](int i) { return frag((i & 1) ? V : K, jt * 32, plr, (i >> 1) * 16 + g * 8); };
#pragma unroll
          for (int i = 0; i < RING; ++i) fb[i] = fetch(i);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            if (i & 1) dp = mfma(fb[i % RING], dof[i >> 1], dp);
            else s = mfma(fb[i % RING], qf[i >> 1], s);
            if (i + RING < 16) fb[i % RING] = fetch(i + RING);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#endif
        if (diag || edge_q) {   // wave-uniform: only a tile on the diagonal or the last query block needs per-element tests (-4.5 %)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            float p = __builtin_amdgcn_exp2f(s[q] * c - lse_i);
            if (!valid || (diag && (j0 + jt * 32 + acc_row(q, g) > iq))) p = 0.f;
            s[q] = p * (dp[q] - del_i);
          }
        } else {
#pragma unroll
          for (int q = 0; q < 16; ++q) s[q] = __builtin_amdgcn_exp2f(s[q] * c - lse_i) * (dp[q] - del_i);
        }
        dsf[2 * jt] = pack_half(s, 0);
        dsf[2 * jt + 1] = pack_half(s, 1);
      }
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dq[ct] = mfma(frag_tr(K, ks * 16, ct * 32, lane), dsf[ks], dq[ct]);
    }
    TIDE_ATTN_WAIT_DMA();
    __syncthreads();
  }
  stage_out(smem, dq, scale, wave, lane);
  __syncthreads();
  copy_out(smem, dqkv, sv.row0 + q0, sv.row0 + min(S, q0 + BQ), ld, h * D, tid);
}

// ------------------------------------------------------------------------------------------------
// backward, dK and dV
// ------------------------------------------------------------------------------------------------
namespace {
// Query rows per streamed tile (32 or 64: two halves of 32 between two barriers) of the dV and of the dK pass.
// Measured, backward at 16 x 2048 / 2 x 16384 (dV rows / dK rows): 32 / 32: 3.18 / 18.2 ms; 32 / 64: 3.08 / 18.0;
// 64 / 32: 3.14 / 18.7; 64 / 64: 3.09 / 18.5 (with 64 rows the dV pass loses its third block per CU to the LDS).
#ifndef TIDE_ATTN_DV_ROWS
#define TIDE_ATTN_DV_ROWS 32
#endif
#ifndef TIDE_ATTN_DK_ROWS
#define TIDE_ATTN_DK_ROWS 64
#endif
template <int BI> struct DkvStage {
  static constexpr int Q_TILE = TileDma<BI>::CHUNKS * 512;   // elements: the tile rounded up to whole 1 KiB chunks of the LDS-DMA loads
  static constexpr int STAGE = 2 * Q_TILE + 4 * BI;          // Q tile, dO tile, then lse[BI] and delta[BI] as floats
};
}  // namespace

// One gradient per pass (WHICH = 0: dV, 1: dK).  Half the accumulators and, for dV, half the operand
// registers of the fused kernel: the pass fits 256 VGPRs, two blocks share a CU, and one block's
// exponentials overlap the other's MFMAs.  The price is that S = Q K^T is computed in both passes.
template <int WHICH>
__global__ __launch_bounds__(256, (WHICH == 0 ? 3 : 2)) void attn_dkv_mfma_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            bf16_t* __restrict__ dqkv, int Smax, int nh, int nkv,
                                                            const int* __restrict__ cu, int64_t T, int nseq) {
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5, plr = perm(lr);
  const Work3 wk = xcd_group_work((Smax + 127) / 128, nkv, nseq, 1);
  const int jb = wk.x, kh = wk.y, b = wk.z;  // early key blocks are the heavy ones
  const SeqView sv = seq_view(cu, b, Smax, T);
  const int S = sv.len;
  const int G = nh / nkv;
  const int ld = (nh + 2 * nkv) * D, ldo = nh * D;
  const int j0 = jb * 128, jw = j0 + wave * 32, jk = jw + lr;
  if (j0 >= S) return;   // the whole block, before any barrier
  const __amdgpu_buffer_rsrc_t rs = rsrc(qkv + (size_t)sv.row0 * ld, (uint32_t)((size_t)S * ld * 2));
  const int kcol = (nh + kh) * D, vcol = (nh + nkv + kh) * D;
  const float scale = 1.0f / sqrtf((float)D);
  const float c = kLog2e * scale;

  constexpr bool DK = WHICH == 1;
  constexpr int BI = DK ? TIDE_ATTN_DK_ROWS : TIDE_ATTN_DV_ROWS;
  constexpr int Q_TILE = DkvStage<BI>::Q_TILE, DKV_STAGE = DkvStage<BI>::STAGE;
  u32x4_t kf[8], vf[DK ? 8 : 1];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    kf[kk] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, ((uint32_t)jk * (uint32_t)ld + (uint32_t)(kcol + kk * 16 + g * 8)) * 2u, 0, 0));
    if constexpr (DK) vf[kk] = __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, ((uint32_t)jk * (uint32_t)ld + (uint32_t)(vcol + kk * 16 + g * 8)) * 2u, 0, 0));
  }
  f32x16_t dacc[4];   // dK or dV of this wave's 32 keys
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int q = 0; q < 16; ++q) dacc[ct][q] = 0.f;

  const int i_begin = (j0 / BI) * BI;                  // first query tile that can see a key of this block
  const int nit = (S - i_begin + BI - 1) / BI;         // query tiles per head
  const int ntiles = G * nit;

  const i32x4_t rsq = rsrc_words(qkv + (size_t)sv.row0 * ld, (uint32_t)((size_t)S * ld * 2));
  const i32x4_t rsdo = rsrc_words(dout + (size_t)sv.row0 * ldo, (uint32_t)((size_t)S * ldo * 2));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  TileDma<BI> dmq, dmo;   // LDS-DMA loads of the Q and the dO tile (their row pitches in memory differ)
  dmq.init(ld, wave, lane);
  dmo.init(ldo, wave, lane);
  float stat = 0.f;  // threads 0..BI-1 carry lse, BI..2BI-1 carry delta of the staged tile
  // Query tiles are walked from the END of the sequence down to the first one that sees this block's keys: the key
  // blocks of a kv head run side by side on one XCD, and this way all of them want the same Q / dO tile at about
  // the same time (walking up from each block's own first tile, they were spread over the whole sequence and the
  // passes fetched nearly every tile through the fabric: 3.8 GB per launch at the 8B shape, L2 hits 21 %).
  // (and tile by tile over the G query heads, not head by head: blocks with fewer tiles would otherwise move on
  // to the next head early)
  auto tile_i0 = [&](int u) { return i_begin + (nit - 1 - u / G) * BI; };
  auto gload = [&](int u, int st) {   // tile u into stage st (whose last readers have passed a barrier)
    const int hh = kh * G + u % G;
    const int i0 = tile_i0(u);
    bf16_t* base = smem + st * DKV_STAGE;
    dmq.issue(rsq, base, ((uint32_t)i0 * (uint32_t)ld + (uint32_t)(hh * D)) * 2u, wave_s);
    dmo.issue(rsdo, base + Q_TILE, ((uint32_t)i0 * (uint32_t)ldo + (uint32_t)(hh * D)) * 2u, wave_s);
    if (tid < 2 * BI) {
      const int i = i0 + (tid & (BI - 1));
      const float* src = (tid < BI) ? lse : delta;
      // (used in sstore only: the load stays in flight; a row past the sequence gets lse = +inf there, delta = 0)
      stat = (i < S) ? src[stat_index(cu, T, sv, b, hh, nh, Smax, i)] : ((tid < BI) ? INFINITY : 0.f);
    }
  };
  auto sstore = [&](int st) {
    bf16_t* base = smem + st * DKV_STAGE;
    if (tid < 2 * BI) reinterpret_cast<float*>(base + 2 * Q_TILE)[tid] = stat * ((tid < BI) ? kLog2e : 1.f);   // lse * log2(e), delta
  };

  gload(0, 0);
  sstore(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the tile and the K / V fragments have arrived before the loop
  __syncthreads();
  for (int u = 0; u < ntiles; ++u) {
    const int st = u & 1;
    if (u + 1 < ntiles) gload(u + 1, st ^ 1);
    const int it0 = tile_i0(u);
#pragma unroll
    for (int hf = 0; hf < BI / 32; ++hf) {
    const int i0 = it0 + hf * 32;   // this half's first query
    if (i0 + 31 >= jw && i0 < S) {  // wave-uniform: some query of the half sees some key of this wave
      const bf16_t* Qt = smem + st * DKV_STAGE;
      const bf16_t* dOt = Qt + Q_TILE;
      const float* stats = reinterpret_cast<const float*>(Qt + 2 * Q_TILE) + hf * 32;
      f32x16_t s, dp;
#pragma unroll
      for (int q = 0; q < 16; ++q) { s[q] = 0.f; dp[q] = 0.f; }
      {
        // Q (and, in the dK pass, dO) fragments through a ring, each requested TIDE_ATTN_DKV_RING MFMAs ahead
        constexpr int RING = TIDE_ATTN_DKV_RING, NF = DK ? 16 : 8;
        u32x4_t fb[RING];
        auto fetch = [&](int i) {
          if constexpr (DK) return frag((i & 1) ? dOt : Qt, hf * 32, plr, (i >> 1) * 16 + g * 8);
          else return frag(Qt, hf * 32, plr, i * 16 + g * 8);
        };
#pragma unroll
        for (int i = 0; i < RING; ++i) fb[i] = fetch(i);
#pragma unroll
        for (int i = 0; i < NF; ++i) {
          if constexpr (DK) {
            if (i & 1) dp = mfma(fb[i % RING], vf[i >> 1], dp);
            else s = mfma(fb[i % RING], kf[i >> 1], s);
          } else {
            s = mfma(fb[i % RING], kf[i], s);
          }
          if (i + RING < NF) fb[i % RING] = fetch(i + RING);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // Rows past the end of the sequence carry lse = +inf (see sstore), i.e. p = 0 without a test; the causal test is
      // per element, and only a half that touches the diagonal makes it (wave-uniform branch).
      const bool diag = i0 < jw + 32;  // some (query, key) pair of the half is above the diagonal
      auto probs = [&](auto MASK) {
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
          const float4 l4 = *reinterpret_cast<const float4*>(stats + 8 * qq + 4 * g);   // lse * log2(e), see sstore
          const float4 d4 = *reinterpret_cast<const float4*>(stats + BI + 8 * qq + 4 * g);
          const float lv4[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int q = qq * 4 + e;
            float p = __builtin_amdgcn_exp2f(s[q] * c - lv4[e]);
            if constexpr (decltype(MASK)::value) {
              if (i0 + 8 * qq + 4 * g + e < jk) p = 0.f;
            }
            s[q] = DK ? p * (dp[q] - dv4[e]) : p;   // dS for the dK pass, P for the dV pass
          }
        }
      };
      if (diag) probs(std::true_type{});
      else probs(std::false_type{});
      const u32x4_t pf[2] = {pack_half(s, 0), pack_half(s, 1)};
      const bf16_t* Xt = DK ? Qt : dOt;   // dK += dS^T Q, dV += P^T dO
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) dacc[ct] = mfma(frag_tr(Xt, hf * 32 + ks * 16, ct * 32, lane), pf[ks], dacc[ct]);
    }
    }
    if (u + 1 < ntiles) sstore(st ^ 1);
    TIDE_ATTN_WAIT_DMA();
    __syncthreads();
  }
  const int64_t r0 = sv.row0 + j0, r1 = sv.row0 + min(S, j0 + 128);
  stage_out(smem, dacc, DK ? scale : 1.0f, wave, lane);
  __syncthreads();
  copy_out(smem, dqkv, r0, r1, ld, DK ? kcol : vcol, tid);
}


// ------------------------------------------------------------------------------------------------
bool attn_mfma_supported(const AttnArgs& a) {
  if (a.dtype != kBF16 || a.dh != D) return false;
  if (a.B <= 0 || a.S <= 0 || a.B > 65535 || a.nh > 65535) return false;
  const int64_t ld = (int64_t)(a.nh + 2 * a.nkv) * D;
  if ((int64_t)a.S * ld * 2 >= ((int64_t)1 << 31)) return false;   // 32-bit offsets inside one sequence
  if (((uintptr_t)a.qkv | (uintptr_t)a.out | (uintptr_t)a.dout | (uintptr_t)a.dqkv) & 15) return false;
  if ((int64_t)((a.S + BQ - 1) / BQ) * a.nh * a.B >= ((int64_t)1 << 31)) return false;   // 1-D grids
  return true;
}

namespace {
constexpr size_t kFwdSmem = (size_t)4 * KV_TILE * sizeof(bf16_t);           // 69632 B (>= the 128 x PITCH output tile)
constexpr size_t kOutTile = (size_t)128 * PITCH * sizeof(bf16_t);
constexpr size_t dkv_smem(int bi) {
  const size_t st = (size_t)2 * (bi == 64 ? DkvStage<64>::STAGE : DkvStage<32>::STAGE) * sizeof(bf16_t);
  return st > kOutTile ? st : kOutTile;
}
constexpr size_t kDvSmem = dkv_smem(TIDE_ATTN_DV_ROWS), kDkSmem = dkv_smem(TIDE_ATTN_DK_ROWS);

hipError_t set_smem(const void* f, size_t bytes, bool& done) {
  if (done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) done = true;
  return e;
}
}  // namespace

hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t s) {
  static bool done = false;
  hipError_t e = set_smem((const void*)attn_fwd_mfma_kernel, kFwdSmem, done);
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)((int64_t)((a.S + BQ - 1) / BQ) * a.nh * a.B));   // 1-D: the kernel maps blocks to work itself
  ProfScope ps("attn_fwd_mfma", 2.0 * a.B * a.nh * D * (double)a.S * (a.S + 1), 0, s);
  hipLaunchKernelGGL(attn_fwd_mfma_kernel, grid, dim3(256), kFwdSmem, s, (const bf16_t*)a.qkv, (bf16_t*)a.out, a.lse, a.S, a.nh, a.nkv, a.cu_seqlens, a.total_rows, a.B);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t s) {
  static bool done_q = false;
  hipError_t e = launch_attn_delta(a, s);
  if (e != hipSuccess) return e;
  e = set_smem((const void*)attn_dq_mfma_kernel, kFwdSmem, done_q);
  if (e != hipSuccess) return e;
  const dim3 gq((unsigned)((int64_t)((a.S + BQ - 1) / BQ) * a.nh * a.B)), gkv((unsigned)((int64_t)((a.S + 127) / 128) * a.nkv * a.B));
  const double pairs = (double)a.B * a.nh * D * (double)a.S * (a.S + 1) / 2.0;  // (query, key, channel) triples
  {
    ProfScope ps("attn_dq_mfma", 6.0 * pairs, 0, s);   // S, dP and dQ products
    hipLaunchKernelGGL(attn_dq_mfma_kernel, gq, dim3(256), kFwdSmem, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse, a.delta, (bf16_t*)a.dqkv, a.S, a.nh, a.nkv, a.cu_seqlens, a.total_rows, a.B);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  static bool done_v = false, done_k = false;
  e = set_smem((const void*)attn_dkv_mfma_kernel<0>, kDvSmem, done_v);
  if (e != hipSuccess) return e;
  e = set_smem((const void*)attn_dkv_mfma_kernel<1>, kDkSmem, done_k);
  if (e != hipSuccess) return e;
  ProfScope ps("attn_dkv_mfma", 10.0 * pairs, 0, s);   // dV pass: S, dV; dK pass: S, dP, dK
  hipLaunchKernelGGL(attn_dkv_mfma_kernel<0>, gkv, dim3(256), kDvSmem, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse, a.delta, (bf16_t*)a.dqkv, a.S, a.nh, a.nkv, a.cu_seqlens, a.total_rows, a.B);
  hipLaunchKernelGGL(attn_dkv_mfma_kernel<1>, gkv, dim3(256), kDkSmem, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse, a.delta, (bf16_t*)a.dqkv, a.S, a.nh, a.nkv, a.cu_seqlens, a.total_rows, a.B);
  return hipGetLastError();
}

}  // namespace tide

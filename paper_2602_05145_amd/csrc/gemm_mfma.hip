// bf16 MFMA GEMM for gfx950 (CDNA4), fp32 accumulation, for the three layouts of the training step:
//   NT  C = A[M,K] B[N,K]^T   forward projections           (both operands K-contiguous)
//   NN  C = A[M,K] B[K,N]     input gradients dX = dY W     (B is N-contiguous)
//   TN  C = A[K,M]^T B[K,N]   weight gradients dW = dY^T X  (both operands contracted over rows)
//
// Design
//   * A block computes a BM x BN tile (256x256 with 8 wavefronts = 2 per SIMD, or 128x128 with 4) with
//     v_mfma_f32_32x32x16_bf16; a wave owns TM x TN MFMA tiles (4x2 or 2x2).  Two waves per SIMD matter:
//     one wave alone cannot issue MFMAs back to back (measured ~83 % of the multi-wave MFMA rate), and a
//     four-wave 256x256 variant (128x128 per wave, a third less LDS read traffic) is slower: 10-20 % under the
//     compiler's schedule, and still 2.5 % (NT), 3 % (NN) and 8 % (TN) with the pinned schedule of the
//     16x16x32 kernel below (its WAVES_N = 2 instantiation: 256 accumulator registers in AGPRs, no spills).
//   * K is walked in slabs through an LDS ring that always holds 128 k-columns and is filled by LDS-DMA
//     buffer loads (global -> LDS without passing through registers, hardware zero-fill outside the valid
//     extent, so ragged M / N / K need no special code).  What bounds this kernel is the memory side: with
//     every operand row aliased to one line (all loads hit) the same code runs 25-40 % faster.  The ring
//     shape of the 32x32x16 kernel follows the operand layout: with a K-major operand the slab is 64 deep
//     (TWO stages): each of its rows then fetches one whole 128-byte line instead of two 64-byte halves;
//     when both operands are row-major over K (TN) their rows are contiguous anyway and FOUR stages of 32
//     win because the loads of slab k+3 are issued while slab k is multiplied.  The 16x16x32 kernel (the
//     one the large launches use) walks slabs of 64 through five units in every layout (see there).
//   * Synchronisation is manual: one `s_waitcnt vmcnt(n)` (own DMA of the next slab has landed, younger
//     slabs stay in flight) and one `s_barrier` per slab.  Each stage is its own __shared__ array and every
//     read address is "array + per-lane offset + constant": the compiler can then tell that the operand
//     reads do not alias the DMA writes in flight and does not drain vmcnt before them (it loses that
//     information on address chains more than a few steps long, and then silently waits).  Slabs past K
//     are dummies (their loads fall outside the buffer and zero-fill the free stage) so the steady state
//     has no branches.
//   * The two-stage loop is software-pipelined across slabs: the barrier of a slab sits before its last
//     k16 quarter, when every wave holds that quarter's operands in registers; the DMA of slab k+2 and the
//     first operand reads of slab k+1 are issued in the shadow of that quarter's MFMAs.
//   * Instruction order inside a k16 quarter is pinned with sched_group_barrier: MFMA / LDS read (or DMA
//     issue) alternate, so LDS and address traffic hides in the MFMA shadow.
//   * LDS layout.  A "K-major" operand (contraction index contiguous in memory) is stored [row][BK] with
//     the 16-byte pieces of a row XOR-swizzled by (row >> 1) & 7 (BK 64) or (row >> 2) & 3 (BK 32): DMA can
//     only write 1 KiB contiguous per instruction, so padding is impossible, and the swizzle makes the
//     16-byte operand reads of 16 consecutive rows hit 16 different bank groups.  An operand whose
//     contraction index is the slow one (B of NN, both operands of TN) is stored as in memory, [k][row],
//     and transposed on the way to the MFMA by ds_read_b64_tr_b16 (two per MFMA operand: four k each);
//     the pieces of k-row k are XOR-swizzled by (k & 3) << 2 so that the four k-rows of one such read lie
//     in different banks.  No transposed copy of an operand ever exists in HBM.
//   * The contraction may run over two operand pairs back to back (d b = dGate W_gate + dUp W_up), and
//     the epilogue fuses alpha (host and device scalar), a residual add, accumulation into C and the cast.
//     bf16 results without residual/accumulate go through a wave-private LDS patch to leave as 16-byte
//     row segments; everything else is stored straight from the accumulators (128-byte row segments).
//   * Work-groups are renumbered so that each of the 8 XCDs (round-robin dispatch) gets a contiguous
//     range of tiles, walked in groups of 4 tile-rows: neighbouring tiles share A/B panels in that
//     XCD's L2.
#include <type_traits>
#include <utility>

#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_vp;

namespace {


struct MfmaParams {
  const bf16_t* A; const bf16_t* B; const bf16_t* A2; const bf16_t* B2;
  void* C; const void* R; const float* alpha_dev;
  int M, N, K, K2;
  int lda, ldb, ldc, ldr;
  float alpha;
  int accumulate;
  int tiles_m, tiles_n;
  const int* m_dev; int m_off;   // optional device-side M: effective M = clamp(*m_dev - m_off, 0, M)
  const int* k_dev; int k_off;   // optional device-side K (pair 0 only)
  // Split of the last, partly filled round of tiles over K (fp32 results only): tiles [0, split_full) are whole;
  // each later tile is worked on by split_s blocks, each over 1/split_s of the slabs; part 0 writes C, part
  // j > 0 writes its 256 x 256 partial sum to split_scratch[(j - 1) * (tiles - split_full) + tile - split_full],
  // and splitk_fixup_kernel adds the partial sums to C in a fixed order afterwards.  split_s <= 1: no split.
  int split_s, split_full;
  float* split_scratch;
};

// tile index (XCD-contiguous order, groups of 4 tile rows) -> tile coordinates
#ifndef TIDE_TILE_GROUP
#define TIDE_TILE_GROUP 4
#endif
__device__ __forceinline__ void tile_coords(int v, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int GROUP = TIDE_TILE_GROUP;
  const int per_group = GROUP * tiles_n;
  const int gid = v / per_group;
  const int first_m = gid * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int in_g = v - gid * per_group;
  tile_m = first_m + in_g % gsz;
  tile_n = in_g / gsz;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// wait until at most n of this wave's vector-memory operations are outstanding (vmcnt only)
#define TIDE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// swizzle of a row-major stage: 16-byte piece index ^= (k-row & 3) << 2, i.e. the four k-rows that one
// transposing read touches sit in four different 64-byte bank groups.  The 16x16x32 kernel also flips bit 1 of the
// piece index with bit 3 of the k-row: there the 16-lane groups of a read differ in k (by 8 rows) and not in the
// column, and the flip keeps two neighbouring groups on different banks.
#define TIDE_RSWZ(kq) ((kq) << 2)
#define TIDE_RSWZ16(krow) ((((krow) & 3) << 2) ^ ((((krow) >> 3) & 1) << 1))
constexpr uint32_t kOobOffset = 0x7FFFFFF0u;  // beyond any buffer extent used here: the load returns zeros

// One LDS-DMA load of 16 bytes per lane, written as an instruction: the 64 lanes' data go to 1 KiB of LDS at
// `lds_addr` (a scalar), each lane fetches from byte `voff` of the buffer `rsrc` (zeros outside its extent).
// The compiler does not see that this writes LDS, so it never orders an LDS read after it by waiting for every
// load in flight (which it does for the builtin form as soon as it cannot prove that the read and the loads in
// flight touch different arrays, e.g. where paths of the loop merge); all waits on these loads are explicit.
typedef int i32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4_t make_rsrc_words(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)base;
  i32x4_t r;
  r[0] = (int)(uint32_t)a; r[1] = (int)((uint32_t)(a >> 32) & 0xffffu); r[2] = (int)bytes; r[3] = 0x00020000;
  return r;
}
__device__ __forceinline__ void dma16(i32x4_t rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc));
}

// One operand (A or B) of one block: R rows (BM or BN) of the tile, either K-major or row-major over K.
template <int R, int NW, bool RMAJ, int T, int BK, int MI = 32>   // T = 32-row MFMA tiles per wave along this dimension; BK = slab depth; MI = MFMA tile edge
struct Operand {
  static constexpr int STAGE = R * BK;                                   // elements per stage
  static constexpr int CHUNKS = STAGE * 2 / 1024;                        // 1 KiB DMA instructions per stage
  static constexpr int PER_WAVE = CHUNKS / NW;
  static_assert(CHUNKS % NW == 0 && PER_WAVE >= 1, "DMA chunks must split evenly over the waves");
  static constexpr int PPR = R / 8;                                      // 16-byte pieces per k-row (row-major)
  static constexpr int RPC = 64 / PPR;                                   // k-rows per DMA chunk (row-major)
  static constexpr int KPIECES = BK / 8;                                 // 16-byte pieces per K-major row (4 or 8)
  static constexpr int KROWS = 64 / KPIECES;                             // K-major rows per DMA chunk (16 or 8)
  static constexpr int SWZ_SHIFT = (BK == 32) ? 2 : 1;                   // swizzle: piece ^= (row >> shift) & (KPIECES-1)
  static constexpr int kReadsPerQuarter = RMAJ ? 2 * T : T;              // LDS read instructions per k16 quarter

  // Stateless on purpose: the tile pointers and extents stay plain kernel locals (SGPRs).  Bundling them
  // in a struct with the per-lane offsets made the compiler keep that struct in scratch memory, the
  // buffer descriptors then lived in VGPRs and every DMA load became a waterfall loop.

  // per-lane byte offsets of this wave's DMA chunks, without the k0 term; K-major also yields the 16-byte
  // piece of a row that this lane fetches (swizzled)
  static __device__ __forceinline__ void lane_offsets(int ld, int wave, int lane, uint32_t (&off)[PER_WAVE],
                                                      int (&piece)[PER_WAVE]) {
    if (RMAJ) {
      // chunk = RPC k-rows x (R*2) bytes; LDS slot (krow, s) holds piece s ^ ((krow & 3) << 2) of that k-row
      const int kr = lane / PPR, pc = lane % PPR;
#pragma unroll
      for (int i = 0; i < PER_WAVE; ++i) {
        const int krow = (wave * PER_WAVE + i) * RPC + kr;
        off[i] = (uint32_t)((krow * ld + (pc ^ (MI == 16 ? TIDE_RSWZ16(krow) : TIDE_RSWZ(krow & 3))) * 8) * 2);
        piece[i] = 0;
      }
    } else {
      // chunk = KROWS rows x (BK*2) bytes; LDS slot (row, s) holds piece s ^ swizzle(row) of that row
      const int rl = lane / KPIECES, slot = lane % KPIECES;
#pragma unroll
      for (int i = 0; i < PER_WAVE; ++i) {
        const int row = (wave * PER_WAVE + i) * KROWS + rl;
        piece[i] = slot ^ ((row >> SWZ_SHIFT) & (KPIECES - 1));
        off[i] = (uint32_t)((row * ld + piece[i] * 8) * 2);
      }
    }
  }

  // Issue the DMA loads of the slab [k0, k0+BK) into `stage`.  tile = operand pointer already offset to
  // the tile's first row (K-major) or first column (row-major); rows_valid = tile rows inside the matrix
  // (K-major) ; cols_left = matrix columns from the tile's first column on (row-major); Kc = contraction
  // length.  A slab with k0 >= Kc is a dummy: every load is out of range and writes zeros.
  static __device__ __forceinline__ void issue(bf16_t* stage, const bf16_t* tile, int ld, int rows_valid, int cols_left,
                                               int k0, int Kc, const uint32_t (&off)[PER_WAVE],
                                               const int (&piece)[PER_WAVE], int wave) {
    if (RMAJ) {
      const int kv = min(BK, Kc - k0);   // valid k-rows of this slab (<= 0 for a dummy slab)
      const bf16_t* base = tile + (size_t)(kv > 0 ? k0 : 0) * ld;
      const uint32_t bytes = kv > 0 ? (uint32_t)(((int64_t)(kv - 1) * ld + cols_left) * 2) : 0u;
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, bytes);
#pragma unroll
      for (int i = 0; i < PER_WAVE; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_vp)(stage + (wave * PER_WAVE + i) * 512), 16, off[i], 0, 0, 0);
    } else {
      const uint32_t bytes = (uint32_t)(((int64_t)(rows_valid - 1) * ld + Kc) * 2);
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(tile, bytes);
#pragma unroll
      for (int i = 0; i < PER_WAVE; ++i) {
        const bool kin = (k0 + piece[i] * 8) < Kc;
        const uint32_t o = kin ? off[i] + (uint32_t)(k0 * 2) : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_vp)(stage + (wave * PER_WAVE + i) * 512), 16, o, 0, 0, 0);
      }
    }
  }

  // The same loads issued one by one as instructions (dma16): slab_desc is the scalar part of a slab, chunk<I>
  // issues the wave's I-th chunk into the LDS unit at byte address `unit` (scalar); wave_s is the wave index as a scalar.
  struct SlabDesc { i32x4_t rs; int k0, Kc; };
  static __device__ __forceinline__ SlabDesc slab_desc(const bf16_t* tile, int ld, int rows_valid, int cols_left, int k0, int Kc) {
    SlabDesc d;
    d.k0 = k0; d.Kc = Kc;
    if (RMAJ) {
      const int kv = min(BK, Kc - k0);
      const bf16_t* base = tile + (size_t)(kv > 0 ? k0 : 0) * ld;
      d.rs = make_rsrc_words(base, kv > 0 ? (uint32_t)(((int64_t)(kv - 1) * ld + cols_left) * 2) : 0u);
    } else {
      d.rs = make_rsrc_words(tile, (uint32_t)(((int64_t)(rows_valid - 1) * ld + Kc) * 2));
    }
    return d;
  }
  // A load whose lane offset is a loop constant: a row-major operand always, a K-major one when every slab is
  // whole (K a multiple of BK), where neither the per-lane test "is this piece still inside K" nor a per-lane k
  // offset is needed: the slab's k0 sits in the descriptor's base (and its extent ends k0 earlier, so the row
  // bound stays where it was), and a dummy slab has an empty extent.
  template <int I>
  static __device__ __forceinline__ void chunk_whole(const SlabDesc& d, uint32_t unit, const uint32_t (&off)[PER_WAVE], int wave_s) {
    dma16(d.rs, unit + (uint32_t)((wave_s * PER_WAVE + I) * 1024), off[I]);
  }
  template <int I>
  static __device__ __forceinline__ void chunk(const SlabDesc& d, uint32_t unit, const uint32_t (&off)[PER_WAVE],
                                               const int (&piece)[PER_WAVE], int wave_s) {
    const uint32_t lds = unit + (uint32_t)((wave_s * PER_WAVE + I) * 1024);
    if (RMAJ) {
      dma16(d.rs, lds, off[I]);
    } else {
      const bool kin = (d.k0 + piece[I] * 8) < d.Kc;
      dma16(d.rs, lds, kin ? off[I] + (uint32_t)(d.k0 * 2) : kOobOffset);
    }
  }

  // Per-lane element offsets of the operand reads inside a stage, computed once.  K-major: one per k16
  // step (the swizzle is an XOR, not additive in the step); row-major: one per MFMA tile.  The values are
  // made opaque to the optimiser: every read address is then "stage array + offset + constant", a short
  // chain that keeps the no-alias information of the stage arrays (longer chains lose it, and a read
  // without it waits for all DMA writes in flight).
  static constexpr int NRO = RMAJ ? T : BK / 16;
  static __device__ __forceinline__ void read_offsets(int wbase, int lane, uint32_t (&ro)[NRO]) {
    const int lr = lane & 31, lg = lane >> 5;
    if (RMAJ) {
      // transposing LDS reads: a group of 16 lanes addresses 4 k-rows x 16 tile rows (lane j: k-row j / 4,
      // rows 4 * (j % 4) .. +3) and lane i of the group receives tile row i for those 4 k
      const int hb = (lane >> 4) & 1, kq = (lane >> 2) & 3, rq = lane & 3;
#pragma unroll
      for (int i = 0; i < T; ++i) {
        const int col = wbase + 32 * i + 16 * hb + 4 * rq;
        ro[i] = (uint32_t)((lg * 8 + kq) * R + ((((col >> 3) ^ TIDE_RSWZ(kq)) << 3) | (col & 7)));
      }
    } else {
      const int sw = (lr >> SWZ_SHIFT) & (KPIECES - 1);
#pragma unroll
      for (int kk = 0; kk < NRO; ++kk) ro[kk] = (uint32_t)((wbase + lr) * BK + (((kk * 2 + lg) ^ sw) * 8));
    }
#pragma unroll
    for (int i = 0; i < NRO; ++i) asm("" : "+v"(ro[i]));
  }

  // ---- 16x16x32 MFMA: a fragment is 16 tile rows x 32 k; lane l holds row l & 15, k = 8 * (l >> 4) .. + 7 ----
  static constexpr int T16 = 2 * T;                          // 16-row fragments per wave along this dimension
  static constexpr int NRO16 = RMAJ ? T16 : BK / 32;
  static constexpr int kReadsPerFrag16 = RMAJ ? 2 : 1;
  static __device__ __forceinline__ void read_offsets16(int wbase, int lane, uint32_t (&ro)[NRO16]) {
    const int r16 = lane & 15, g = lane >> 4;
    if (RMAJ) {
      // transposing reads: lane j of a 16-lane group addresses k-row j / 4, tile rows 4 * (j % 4) .. + 3 and
      // receives tile row j for those 4 k; the group's k-rows start at 8 * g
      const int kq = (lane >> 2) & 3, rq = lane & 3;
#pragma unroll
      for (int i = 0; i < T16; ++i) {
        const int col = wbase + 16 * i + 4 * rq;
        const int krow = g * 8 + kq;
        ro[i] = (uint32_t)(krow * R + ((((col >> 3) ^ TIDE_RSWZ16(krow)) << 3) | (col & 7)));
      }
    } else {
      const int sw = (r16 >> SWZ_SHIFT) & (KPIECES - 1);
#pragma unroll
      for (int h = 0; h < NRO16; ++h) ro[h] = (uint32_t)((wbase + r16) * BK + (((h * 4 + g) ^ sw) * 8));
    }
#pragma unroll
    for (int i = 0; i < NRO16; ++i) asm("" : "+v"(ro[i]));
  }
  // NF fragments starting at fragment index F0, of the k32 step `h` (< BK/32) of a stage
  template <int F0, int NF, typename StagePtr>
  static __device__ __forceinline__ void frags16(StagePtr stage, int h, const uint32_t (&ro)[NRO16], u32x4_t (&f)[NF]) {
    if (RMAJ) {
      typedef short s16x4_t __attribute__((ext_vector_type(4)));
      typedef __attribute__((address_space(3))) s16x4_t* lds_tr_t;
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_t)(stage + ro[F0 + i] + (h * 32) * R));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_t)(stage + ro[F0 + i] + (h * 32 + 4) * R));
        const uint2 a = __builtin_bit_cast(uint2, lo), b2 = __builtin_bit_cast(uint2, hi);
        f[i][0] = a.x; f[i][1] = a.y; f[i][2] = b2.x; f[i][3] = b2.y;
      }
    } else {
      typedef __attribute__((address_space(3))) const u32x4_t* lds_v4_t;
#pragma unroll
      for (int i = 0; i < NF; ++i) f[i] = *(lds_v4_t)(stage + ro[h] + (F0 + i) * 16 * BK);
    }
  }

  // MFMA operand fragments of k16 step `kk` (< BK/16)
  template <typename StagePtr>
  static __device__ __forceinline__ void frags(StagePtr stage, int kk, const uint32_t (&ro)[NRO], u32x4_t (&f)[T]) {
    if (RMAJ) {
      typedef short s16x4_t __attribute__((ext_vector_type(4)));
      typedef __attribute__((address_space(3))) s16x4_t* lds_tr_t;
#pragma unroll
      for (int i = 0; i < T; ++i) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_t)(stage + ro[i] + (kk * 16) * R));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_t)(stage + ro[i] + (kk * 16 + 4) * R));
        const uint2 a = __builtin_bit_cast(uint2, lo), b2 = __builtin_bit_cast(uint2, hi);
        f[i][0] = a.x; f[i][1] = a.y; f[i][2] = b2.x; f[i][3] = b2.y;
      }
    } else {
      typedef __attribute__((address_space(3))) const u32x4_t* lds_v4_t;
#pragma unroll
      for (int i = 0; i < T; ++i) f[i] = *(lds_v4_t)(stage + ro[kk] + i * 32 * BK);
    }
  }
};

template <int N>
struct Int : std::integral_constant<int, N> {};

// Pin the instruction order of one k16 quarter: after MFMA number I come its share of NDS LDS reads and
// of NVM DMA issues.
template <int I, int NMF, int NDS, int NVM, int SYNC>
__device__ __forceinline__ void sched_slot() {
  __builtin_amdgcn_sched_group_barrier(0x008, 1, SYNC);   // MFMA
  constexpr int nds = NDS / NMF + (I < NDS % NMF ? 1 : 0);
  if constexpr (nds > 0) __builtin_amdgcn_sched_group_barrier(0x100, nds, SYNC);   // LDS reads
  constexpr int nvm = NVM / NMF + (I < NVM % NMF ? 1 : 0);
  if constexpr (nvm > 0) __builtin_amdgcn_sched_group_barrier(0x020, nvm, SYNC);   // DMA issues
}
template <int NMF, int NDS, int NVM, int SYNC, int... I>
__device__ __forceinline__ void sched_slots(std::integer_sequence<int, I...>) {
  (sched_slot<I, NMF, NDS, NVM, SYNC>(), ...);
}

}  // namespace

template <int BM, int BN, int NW, bool AMM, bool BNM, typename TO, int BK>
__global__ __launch_bounds__(NW * 64) void gemm_mfma_kernel(MfmaParams p) {
  static_assert(BK == 32 || BK == 64, "slab depth");
  constexpr int NST = (BK == 32) ? 4 : 2;   // LDS stages: the ring always holds 128 k-columns
  constexpr int WAVES_N = (NW == 8) ? 4 : 2, WAVES_M = NW / WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM == 4 || TM == 2, "wave tile height must be 128 or 64");
  static_assert(TN == 4 || TN == 2, "wave tile width must be 128 or 64");
  using OpA = Operand<BM, NW, AMM, TM, BK>;
  using OpB = Operand<BN, NW, BNM, TN, BK>;
  constexpr int A_STAGE = OpA::STAGE, B_STAGE = OpB::STAGE;
  constexpr int NVM = OpA::PER_WAVE + OpB::PER_WAVE;            // DMA instructions per wave per slab
  constexpr int NDS = OpA::kReadsPerQuarter + OpB::kReadsPerQuarter;  // LDS reads per wave per k16 quarter
  constexpr int NMF = TM * TN;                                        // MFMAs per wave per k16 quarter

  constexpr int STAGE34 = (NST == 4) ? A_STAGE + B_STAGE : 8;   // stages 2, 3 exist only in the four-stage ring
  __shared__ __attribute__((aligned(1024))) bf16_t s0[A_STAGE + B_STAGE];
  __shared__ __attribute__((aligned(1024))) bf16_t s1[A_STAGE + B_STAGE];
  __shared__ __attribute__((aligned(1024))) bf16_t s2[STAGE34];
  __shared__ __attribute__((aligned(1024))) bf16_t s3[STAGE34];
  auto stage = [&](auto ST) -> bf16_t* {
    if constexpr (decltype(ST)::value == 0) return s0;
    else if constexpr (decltype(ST)::value == 1) return s1;
    else if constexpr (decltype(ST)::value == 2) return s2;
    else return s3;
  };
  typedef __attribute__((address_space(3))) const bf16_t* lds_bf_t;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lr = lane & 31, lg = lane >> 5;

  // sizes that are only known on the device (block-uniform)
  if (p.m_dev) p.M = max(0, min(p.M, *p.m_dev - p.m_off));
  if (p.k_dev) p.K = max(0, min(p.K, *p.k_dev - p.k_off));
  if (p.K == 0 && p.K2 == 0 && p.accumulate) return;   // nothing to add

  // ---- XCD-aware tile numbering over the tiles that exist for the effective M ----
  int tile_m, tile_n;
  {
    const int tiles_m = (p.M + BM - 1) / BM;   // <= p.tiles_m, the grid's worst case
    const int nb = tiles_m * p.tiles_n;
    const int pid = blockIdx.x;
    if (pid >= nb) return;                     // whole block, before any barrier
    const int xcd = pid & 7, idx = pid >> 3;
    const int q = nb >> 3, r = nb & 7;
    const int v = xcd * q + min(xcd, r) + idx;  // contiguous range per XCD
    constexpr int GROUP = 4;   // 4 tile rows x 8 tile columns per XCD round measured best (8 x 4: +0.8 %, 16 x 2: +4 %, 2 x 16: +1 % step time)
    const int per_group = GROUP * p.tiles_n;
    const int gid = v / per_group;
    const int first_m = gid * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_g = v - gid * per_group;
    tile_m = first_m + in_g % gsz;
    tile_n = in_g / gsz;
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // tile pointers of both operand pairs (uniform) and this lane's DMA offsets
  const bf16_t* a_tile0 = AMM ? p.A + m0 : p.A + (size_t)m0 * p.lda;
  const bf16_t* b_tile0 = BNM ? p.B + n0 : p.B + (size_t)n0 * p.ldb;
  const bf16_t* a_tile1 = p.A2 ? (AMM ? p.A2 + m0 : p.A2 + (size_t)m0 * p.lda) : a_tile0;
  const bf16_t* b_tile1 = p.B2 ? (BNM ? p.B2 + n0 : p.B2 + (size_t)n0 * p.ldb) : b_tile0;
  const int a_rows = min(BM, p.M - m0), b_rows = min(BN, p.N - n0);
  uint32_t a_off[OpA::PER_WAVE], b_off[OpB::PER_WAVE];
  int a_piece[OpA::PER_WAVE], b_piece[OpB::PER_WAVE];
  OpA::lane_offsets(p.lda, wave, lane, a_off, a_piece);
  OpB::lane_offsets(p.ldb, wave, lane, b_off, b_piece);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  const int nk1 = (p.K + BK - 1) / BK;
  const int nkp2 = p.A2 ? (p.K2 + BK - 1) / BK : 0;
  const int nk = nk1 + nkp2;
  const int nk_round = (nk + NST - 1) / NST * NST;   // slabs past nk are dummies

  auto issue = [&](auto ST, int kt) {
    bf16_t* sb = stage(ST);
    int pr = 0, k0 = kt * BK, Kc = p.K;
    if (kt >= nk1) {
      if (kt < nk) { pr = 1; k0 = (kt - nk1) * BK; Kc = p.K2; }
      else { k0 = p.K + BK; }   // dummy slab: everything out of range
    }
    OpA::issue(sb, pr ? a_tile1 : a_tile0, p.lda, a_rows, p.M - m0, k0, Kc, a_off, a_piece, wave);
    OpB::issue(sb + A_STAGE, pr ? b_tile1 : b_tile0, p.ldb, b_rows, p.N - n0, k0, Kc, b_off, b_piece, wave);
  };
  uint32_t a_ro[OpA::NRO], b_ro[OpB::NRO];
  OpA::read_offsets(wave_m * WM, lane, a_ro);
  OpB::read_offsets(wave_n * WN, lane, b_ro);
  auto frags = [&](auto ST, int kk, u32x4_t (&fa)[TM], u32x4_t (&fb)[TN]) {
    const lds_bf_t sb = (lds_bf_t)stage(ST);
    OpA::frags(sb, kk, a_ro, fa);
    OpB::frags(sb + A_STAGE, kk, b_ro, fb);
  };
  auto mma = [&](u32x4_t (&fa)[TM], u32x4_t (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[i]),
                                                            __builtin_bit_cast(bf16x8_t, fb[j]), acc[i][j], 0, 0, 0);
  };

  u32x4_t fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  if constexpr (BK == 64) {
    // ---- two stages of 64 ----
    // Software-pipelined across slabs: the single barrier of a step sits before its LAST k16 quarter.  By
    // then every wave holds the operands of that quarter in registers, so the stage is free: the DMA of slab
    // kt+2 is issued into it and the first operands of slab kt+1 are read, both in the shadow of the last
    // quarter's MFMAs.  No MFMA ever waits for an LDS read that was issued after a barrier.
    issue(Int<0>{}, 0);
    TIDE_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(Int<0>{}, 0, fa0, fb0);
    issue(Int<1>{}, 1);
    __builtin_amdgcn_sched_barrier(0);
    // One step: slab kt lives in stage ST (its quarter-0 operands are already in fa0/fb0), slab kt+1 is in
    // flight into SO.
    auto step = [&](auto ST, auto SO, int kt) {
      frags(ST, 1, fa1, fb1);
      mma(fa0, fb0);
      sched_slots<NMF, NDS, 0, 0>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
      frags(ST, 2, fa0, fb0);
      mma(fa1, fb1);
      sched_slots<NMF, NDS, 0, 1>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
      frags(ST, 3, fa1, fb1);
      mma(fa0, fb0);
      sched_slots<NMF, NDS, 0, 2>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
      // all operand reads of this wave from ST have returned; its part of slab kt+1 has landed
      __builtin_amdgcn_s_waitcnt(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      frags(SO, 0, fa0, fb0);
      issue(ST, kt + 2);
      mma(fa1, fb1);
      // all operand reads ahead of the DMA issues: a read that lost its no-alias information on the way
      // through the compiler would otherwise wait for the loads just issued
      __builtin_amdgcn_sched_group_barrier(0x100, NDS, 3);
      sched_slots<NMF, 0, NVM, 3>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
    };
    for (int kt = 0; kt < nk_round; kt += 2) {
      step(Int<0>{}, Int<1>{}, kt);
      step(Int<1>{}, Int<0>{}, kt + 1);
    }
  } else {
    // ---- four stages of 32: used when both operands are row-major over K (their rows are contiguous
    // anyway, so the deeper ring is what helps); the loads of slab k+3 are issued while slab k is multiplied
    issue(Int<0>{}, 0);
    issue(Int<1>{}, 1);
    issue(Int<2>{}, 2);
    TIDE_WAIT_VMCNT(2 * NVM);
    __builtin_amdgcn_s_barrier();
    frags(Int<0>{}, 0, fa0, fb0);
    // One pipeline step: slab kt lives in stage ST, slab kt+1 in SN, and slab kt+3 goes to SP (the stage
    // slab kt-1 just vacated).  The barrier sits between the two k16 halves so that the operand reads of
    // the next slab are issued under the MFMAs of this one.
    auto step = [&](auto ST, auto SN, auto SP, int kt) {
      frags(ST, 1, fa1, fb1);
      issue(SP, kt + NST - 1);
      mma(fa0, fb0);
      sched_slots<NMF, NDS, NVM, 0>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
      TIDE_WAIT_VMCNT(2 * NVM);          // this wave's part of slab kt+1 has landed (two younger slabs in flight)
      __builtin_amdgcn_s_barrier();      // ... and everybody else's; everybody is done reading slab kt-1
      __builtin_amdgcn_sched_barrier(0);
      frags(SN, 0, fa0, fb0);
      mma(fa1, fb1);
      sched_slots<NMF, NDS, 0, 1>(std::make_integer_sequence<int, NMF>{});
      __builtin_amdgcn_sched_barrier(0);
    };
    for (int kt = 0; kt < nk_round; kt += 4) {
      step(Int<0>{}, Int<1>{}, Int<3>{}, kt);
      step(Int<1>{}, Int<2>{}, Int<0>{}, kt + 1);
      step(Int<2>{}, Int<3>{}, Int<1>{}, kt + 2);
      step(Int<3>{}, Int<0>{}, Int<2>{}, kt + 3);
    }
  }
  TIDE_WAIT_VMCNT(0);   // the dummy slabs still in flight write LDS: let them land before the block retires

  // ---- epilogue ----
  float alpha = p.alpha;
  if (p.alpha_dev) alpha *= *p.alpha_dev;
  TO* C = (TO*)p.C;
  const TO* R = (const TO*)p.R;
  const int wm0 = m0 + wave_m * WM, wn0 = n0 + wave_n * WN;

  // MFMA tile (i, j) of the wave: accumulator register q of lane (lr, lg) is row 8*(q/4) + 4*lg + q%4, column lr.
  bool staged = false;
  if constexpr (sizeof(TO) == 2) {
    if (!R && !p.accumulate && (p.ldc % 8) == 0 && (p.N % 8) == 0) {
      staged = true;
      // bf16 result through a wave-private LDS patch so that it leaves as 16-byte row segments.
      // All stages are free here: every wave waited for its own DMA above, and the barrier below orders the
      // (unused) operand reads of the final dummy slab before the patch writes.
      __builtin_amdgcn_s_barrier();
      constexpr int PP = WN + 8;                       // patch pitch (elements)
      static_assert((NW / 2) * 32 * PP <= A_STAGE + B_STAGE, "epilogue patches of half the waves must fit in one stage");
      bf16_t* patch = (wave < NW / 2 ? s0 : s1) + (wave % (NW / 2)) * (32 * PP);   // 32 x WN per wave
      constexpr int PIECES = WN / 8;                   // 16-byte pieces per patch row
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            const int rr = 8 * (q >> 2) + 4 * lg + (q & 3);
            patch[rr * PP + 32 * j + lr] = f2bf(alpha * acc[i][j][q]);
          }
#pragma unroll
        for (int t = 0; t < 32 * PIECES / 64; ++t) {
          const int pc = lane + 64 * t;
          const int row = pc / PIECES, piece = pc % PIECES;
          const int gm = wm0 + 32 * i + row, gn = wn0 + piece * 8;
          const u32x4_t val = *reinterpret_cast<const u32x4_t*>(patch + row * PP + piece * 8);
          if (gm < p.M && gn < p.N)
            *reinterpret_cast<u32x4_t*>(reinterpret_cast<bf16_t*>(C) + (size_t)gm * p.ldc + gn) = val;
        }
      }
    } else if constexpr ((NW / 2) * 32 * (WN + 4) * 2 <= A_STAGE + B_STAGE) {
      if (R && !p.accumulate && (p.ldc % 8) == 0 && (p.ldr % 8) == 0 && (p.N % 8) == 0) {
        staged = true;
        // bf16 result plus residual: the patch keeps fp32 so that alpha*acc + residual is rounded once, as in
        // the direct path; residual and result move as 16-byte row segments.
        __builtin_amdgcn_s_barrier();
        constexpr int PF = WN + 4;                     // patch pitch (floats)
        float* patch = reinterpret_cast<float*>(wave < NW / 2 ? s0 : s1) + (wave % (NW / 2)) * (32 * PF);
        constexpr int PIECES = WN / 8;
        const bf16_t* Rb = reinterpret_cast<const bf16_t*>(R);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
              const int rr = 8 * (q >> 2) + 4 * lg + (q & 3);
              patch[rr * PF + 32 * j + lr] = alpha * acc[i][j][q];
            }
#pragma unroll
          for (int t = 0; t < 32 * PIECES / 64; ++t) {
            const int pc = lane + 64 * t;
            const int row = pc / PIECES, piece = pc % PIECES;
            const int gm = wm0 + 32 * i + row, gn = wn0 + piece * 8;
            if (gm < p.M && gn < p.N) {
              float v[8], r[8];
              const float4 a0 = *reinterpret_cast<const float4*>(patch + row * PF + piece * 8);
              const float4 a1 = *reinterpret_cast<const float4*>(patch + row * PF + piece * 8 + 4);
              v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
              ld8(Rb, (size_t)gm * p.ldr + gn, r);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += r[e];
              st8(reinterpret_cast<bf16_t*>(C), (size_t)gm * p.ldc + gn, v);
            }
          }
        }
      }
    }
  }
  if (!staged && p.accumulate && !R) {
    // C += alpha * acc.  The old values of a 32-row slice are all requested before the first of them is used
    // (32 or 64 loads in flight per lane instead of a load-add-store chain per element: the compiler cannot
    // reorder the loads itself, it does not know that the stores of one element leave the next one alone).
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float old[16][TN];
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int gm = wm0 + 32 * i + 8 * (q >> 2) + 4 * lg + (q & 3);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int gn = wn0 + 32 * j + lr;
          old[q][j] = (gm < p.M && gn < p.N) ? ldf(C, (size_t)gm * p.ldc + gn) : 0.f;
        }
      }
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int gm = wm0 + 32 * i + 8 * (q >> 2) + 4 * lg + (q & 3);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int gn = wn0 + 32 * j + lr;
          if (gm < p.M && gn < p.N) stf(C, (size_t)gm * p.ldc + gn, alpha * acc[i][j][q] + old[q][j]);
        }
      }
    }
  } else if (!staged) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int rr = 8 * (q >> 2) + 4 * lg + (q & 3);
        const int gm = wm0 + 32 * i + rr;
        if (gm >= p.M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int gn = wn0 + 32 * j + lr;
          if (gn >= p.N) continue;
          float v = alpha * acc[i][j][q];
          if (R) v += ldf(R, (size_t)gm * p.ldr + gn);
          if (p.accumulate) v += ldf(C, (size_t)gm * p.ldc + gn);
          stf(C, (size_t)gm * p.ldc + gn, v);
        }
      }
  }
}


// ------------------------------------------------------------------------------------------------
// The 256x256 tile with v_mfma_f32_16x16x32_bf16.  Same ring, DMA, swizzles, synchronisation and epilogues as
// the kernel above; what changes is the matrix instruction: on this chip the matrix pipes sustain a higher rate
// under the package power limit with the 16x16x32 form (a pure-MFMA loop on random operands: 2.10 against 1.88
// PFLOP/s), while the LDS operand traffic per flop stays the same (a 16-row x 32-k fragment is one 16-byte
// read per lane, like a 32-row x 16-k one).  A wave owns 8 x 4 tiles of 16 x 16 (128 x 64); a "quarter" of the
// schedule is one k32 step of four of its A fragments against its four B fragments: 16 MFMAs (256 clocks, as the
// 8 MFMAs of a k16 quarter above), with the A fragments double-buffered per quarter and the B fragments per k32
// step.  The MFMAs take the B fragment first, so accumulator element q of lane l in tile (i, j) is row
// 16 i + (l & 15), column 16 j + 4 (l >> 4) + q (see the epilogue).  WAVES_N = 4 is the layout in use; with
// WAVES_N = 2 the block has four waves of 128 x 128 (one per SIMD), kept as the measured alternative.
// KWHOLE: every slab of the launch is whole (K, and K2 of a second operand pair, multiples of 64 known on the
// host).  A K-major operand's loads then need neither the per-lane test "is this piece still inside K" nor a
// per-lane k offset: k0 moves into the buffer descriptor and the lane offsets are loop constants, which takes
// three vector instructions per load out of the loop (they compete with the MFMAs for the vector issue port;
// NT 33.2 -> 32.2 ms and NN 30.1 -> 29.5 ms per training step at the 8B shape).
// ------------------------------------------------------------------------------------------------
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <bool AMM, bool BNM, typename TO, int BK, int WAVES_N, bool KWHOLE>
__global__ __launch_bounds__(2 * WAVES_N * 64) void gemm_mfma16_kernel(MfmaParams p) {
  constexpr int BM = 256, BN = 256, WAVES_M = 2, NW = WAVES_M * WAVES_N;
  static_assert(BK == 64, "slab depth");
  static_assert(WAVES_N == 4 || WAVES_N == 2, "eight waves of 128 x 64 or four of 128 x 128");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // 128 x 64
  constexpr int TM = WM / 16, TN = WN / 16;             // 8 x 4 tiles of 16 x 16
  constexpr int GA = 4;                                 // A fragments per quarter
  using OpA = Operand<BM, NW, AMM, WM / 32, BK, 16>;
  using OpB = Operand<BN, NW, BNM, WN / 32, BK, 16>;
  constexpr int A_STAGE = OpA::STAGE, B_STAGE = OpB::STAGE;
  constexpr int NVA = OpA::PER_WAVE, NVB = OpB::PER_WAVE;
  constexpr int NMF = GA * TN;                          // MFMAs per quarter
  typedef __attribute__((address_space(3))) const bf16_t* lds_bf_t;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lc = lane & 15, lg = lane >> 4;

  if (p.m_dev) p.M = max(0, min(p.M, *p.m_dev - p.m_off));
  if (p.k_dev) p.K = max(0, min(p.K, *p.k_dev - p.k_off));
  if (p.K == 0 && p.K2 == 0 && p.accumulate && p.split_s <= 1) return;

  int tile_m, tile_n;
  int part = 0, nparts = 1, tail_index = 0;   // K split of the tiles of the last round (see MfmaParams)
  {
    const int tiles_m = (p.M + BM - 1) / BM;
    const int nb = tiles_m * p.tiles_n;
    const bool split = p.split_s > 1;        // (never together with a device-side M: nb is then the grid's count)
    const int items = split ? p.split_full + (nb - p.split_full) * p.split_s : nb;
    int pid = blockIdx.x;
    if (pid >= items) return;
    // Work-groups go to the XCDs round-robin in the order of their index: the whole tiles (a multiple of 256)
    // come first and each XCD gets a contiguous range of them; the parts of the split tiles come last, again
    // spread over all XCDs, so that they fill the last round everywhere.
    int count = split ? p.split_full : nb, base = 0;
    if (split && pid >= p.split_full) { base = p.split_full; pid -= base; count = items - base; }
    const int xcd = pid & 7, idx = pid >> 3;
    const int q = count >> 3, r = count & 7;
    int v = base + xcd * q + min(xcd, r) + idx;
    if (split && v >= p.split_full) {
      const int u = v - p.split_full;
      tail_index = u / p.split_s;
      part = u - tail_index * p.split_s;
      nparts = p.split_s;
      v = p.split_full + tail_index;
    }
    tile_coords(v, tiles_m, p.tiles_n, tile_m, tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const bf16_t* a_tile0 = AMM ? p.A + m0 : p.A + (size_t)m0 * p.lda;
  const bf16_t* b_tile0 = BNM ? p.B + n0 : p.B + (size_t)n0 * p.ldb;
  const bf16_t* a_tile1 = p.A2 ? (AMM ? p.A2 + m0 : p.A2 + (size_t)m0 * p.lda) : a_tile0;
  const bf16_t* b_tile1 = p.B2 ? (BNM ? p.B2 + n0 : p.B2 + (size_t)n0 * p.ldb) : b_tile0;
  const int a_rows = min(BM, p.M - m0), b_rows = min(BN, p.N - n0);
  uint32_t a_off[NVA], b_off[NVB];
  int a_piece[NVA], b_piece[NVB];
  OpA::lane_offsets(p.lda, wave, lane, a_off, a_piece);
  OpB::lane_offsets(p.ldb, wave, lane, b_off, b_piece);

  f32x4_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[i][j][q] = 0.f;

  const int nk1 = (p.K + BK - 1) / BK;
  const int nkp2 = p.A2 ? (p.K2 + BK - 1) / BK : 0;
  // this block's slabs: all of them, or its part of a split tile (slab numbers below are relative to kt_lo)
  const int nk_all = nk1 + nkp2;
  const int per_part = (nk_all + nparts - 1) / nparts;
  const int kt_lo = min(nk_all, part * per_part);
  const int nk = min(nk_all, kt_lo + per_part) - kt_lo;

  // which operand pair and k offset slab kt stands for (slabs past nk are dummies: every load out of range)
  auto slab = [&](int kt, int& pr, int& k0, int& Kc) {
    const int g = kt_lo + kt;
    pr = 0; k0 = g * BK; Kc = p.K;
    if (kt >= nk) { k0 = p.K + BK; }
    else if (g >= nk1) { pr = 1; k0 = (g - nk1) * BK; Kc = p.K2; }
  };
  uint32_t a_ro[OpA::NRO16], b_ro[OpB::NRO16];
  OpA::read_offsets16(wave_m * WM, lane, a_ro);
  OpB::read_offsets16(wave_n * WN, lane, b_ro);
  // A fragments of group G (0, 1) / the B fragments of the k32 step h of an LDS unit
  auto frags_a = [&](const bf16_t* unit, int h, auto G, u32x4_t (&fa)[GA]) {
    OpA::template frags16<decltype(G)::value * GA, GA>((lds_bf_t)unit, h, a_ro, fa);
  };
  auto frags_b = [&](const bf16_t* unit, int h, u32x4_t (&fb)[TN]) {
    OpB::template frags16<0, TN>((lds_bf_t)unit, h, b_ro, fb);
  };
  // ---- epilogue: needs, per wave, an LDS patch of 32 x (WN + 4) floats that no DMA is writing any more ----
  // The MFMAs are issued with their operands swapped (B fragment first), so an accumulator tile holds the
  // TRANSPOSE of its 16 x 16 block: element q of lane l in tile (i, j) is row m = 16 i + (l & 15), columns
  // n = 16 j + 4 (l >> 4) + q.  A lane thus owns four CONSECUTIVE columns of one row: 16 bytes of an fp32 result
  // (one store instead of four), 8 bytes of a bf16 one (one LDS write per tile into the staging patch).
  constexpr int kPatchElems = 32 * (WN + 4) * 2;   // in bf16 elements
  auto epilogue = [&](bf16_t* patch_mem) {
    float alpha = p.alpha;
    if (p.alpha_dev) alpha *= *p.alpha_dev;
    TO* C = (TO*)p.C;
    const TO* R = (const TO*)p.R;
    const int wm0 = m0 + wave_m * WM, wn0 = n0 + wave_n * WN;
    bool staged = false;
    if constexpr (sizeof(TO) == 2) {
      constexpr int PIECES = WN / 8;
      if (!R && !p.accumulate && (p.ldc % 8) == 0 && (p.N % 8) == 0) {
        staged = true;
        // bf16 result through the wave's LDS patch (32 rows = two tile rows at a time) so that it leaves as
        // 16-byte row segments.  Every wave waited for its own DMA; the barrier orders the last operand reads
        // of the other waves before the patch writes.
        __builtin_amdgcn_s_barrier();
        constexpr int PP = WN + 8;
        bf16_t* patch = patch_mem;
#pragma unroll
        for (int i2 = 0; i2 < TM / 2; ++i2) {
#pragma unroll
          for (int ih = 0; ih < 2; ++ih)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const f32x4_t v = acc[2 * i2 + ih][j];
              *reinterpret_cast<uint2*>(patch + (16 * ih + lc) * PP + 16 * j + 4 * lg) =
                  make_uint2(f2bf2(alpha * v[0], alpha * v[1]), f2bf2(alpha * v[2], alpha * v[3]));
            }
#pragma unroll
          for (int t = 0; t < 32 * PIECES / 64; ++t) {
            const int pc = lane + 64 * t;
            const int row = pc / PIECES, piece = pc % PIECES;
            const int gm = wm0 + 32 * i2 + row, gn = wn0 + piece * 8;
            const u32x4_t val = *reinterpret_cast<const u32x4_t*>(patch + row * PP + piece * 8);
            if (gm < p.M && gn < p.N)
              *reinterpret_cast<u32x4_t*>(reinterpret_cast<bf16_t*>(C) + (size_t)gm * p.ldc + gn) = val;
          }
        }
      } else if (R && !p.accumulate && (p.ldc % 8) == 0 && (p.ldr % 8) == 0 && (p.N % 8) == 0) {
        staged = true;
        // bf16 result plus residual: the patch keeps fp32 so that alpha * acc + residual is rounded once
        __builtin_amdgcn_s_barrier();
        constexpr int PF = WN + 4;
        float* patch = reinterpret_cast<float*>(patch_mem);
        const bf16_t* Rb = reinterpret_cast<const bf16_t*>(R);
#pragma unroll
        for (int i2 = 0; i2 < TM / 2; ++i2) {
#pragma unroll
          for (int ih = 0; ih < 2; ++ih)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const f32x4_t v = acc[2 * i2 + ih][j];
              *reinterpret_cast<float4*>(patch + (16 * ih + lc) * PF + 16 * j + 4 * lg) =
                  make_float4(alpha * v[0], alpha * v[1], alpha * v[2], alpha * v[3]);
            }
#pragma unroll
          for (int t = 0; t < 32 * PIECES / 64; ++t) {
            const int pc = lane + 64 * t;
            const int row = pc / PIECES, piece = pc % PIECES;
            const int gm = wm0 + 32 * i2 + row, gn = wn0 + piece * 8;
            if (gm < p.M && gn < p.N) {
              float v[8], r[8];
              const float4 a0 = *reinterpret_cast<const float4*>(patch + row * PF + piece * 8);
              const float4 a1 = *reinterpret_cast<const float4*>(patch + row * PF + piece * 8 + 4);
              v[0] = a0.x; v[1] = a0.y; v[2] = a0.z; v[3] = a0.w; v[4] = a1.x; v[5] = a1.y; v[6] = a1.z; v[7] = a1.w;
              ld8(Rb, (size_t)gm * p.ldr + gn, r);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += r[e];
              st8(reinterpret_cast<bf16_t*>(C), (size_t)gm * p.ldc + gn, v);
            }
          }
        }
      }
    }
    if (staged) return;
    if constexpr (sizeof(TO) == 4) {
      if (!R && (p.ldc % 4) == 0 && (p.N % 4) == 0 && (((uintptr_t)C) & 15) == 0) {
        // fp32 result: a lane's four columns are one 16-byte access.  With accumulate, the old values of two tile
        // rows are all requested before the first of them is used.  A later part of a split tile stores its
        // partial sum to its scratch tile instead (pitch 256, tile-local coordinates, never accumulating).
        float* Cf = reinterpret_cast<float*>(C);
        size_t pitch = (size_t)p.ldc;
        int mo = 0, no = 0;
        bool add = p.accumulate != 0;
        if (part > 0) {
          const int ntail = ((p.M + BM - 1) / BM) * p.tiles_n - p.split_full;
          Cf = p.split_scratch + ((size_t)(part - 1) * ntail + tail_index) * (size_t)(BM * BN);
          pitch = BN; mo = m0; no = n0; add = false;
        }
#pragma unroll
        for (int i2 = 0; i2 < TM / 2; ++i2) {
          float4 old[2][TN];
          if (add) {
#pragma unroll
            for (int ih = 0; ih < 2; ++ih)
#pragma unroll
              for (int j = 0; j < TN; ++j) {
                const int gm = wm0 + 16 * (2 * i2 + ih) + lc, gn = wn0 + 16 * j + 4 * lg;
                old[ih][j] = (gm < p.M && gn < p.N) ? *reinterpret_cast<const float4*>(Cf + (size_t)gm * pitch + gn)
                                                    : make_float4(0.f, 0.f, 0.f, 0.f);
              }
          }
#pragma unroll
          for (int ih = 0; ih < 2; ++ih)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const int gm = wm0 + 16 * (2 * i2 + ih) + lc, gn = wn0 + 16 * j + 4 * lg;
              const f32x4_t v = acc[2 * i2 + ih][j];
              float4 o = make_float4(alpha * v[0], alpha * v[1], alpha * v[2], alpha * v[3]);
              if (add) { o.x += old[ih][j].x; o.y += old[ih][j].y; o.z += old[ih][j].z; o.w += old[ih][j].w; }
              if (gm < p.M && gn < p.N) *reinterpret_cast<float4*>(Cf + (size_t)(gm - mo) * pitch + (gn - no)) = o;
            }
        }
        return;
      }
    }
    // everything else, element by element
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int gm = wm0 + 16 * i + lc;
      if (gm >= p.M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gn = wn0 + 16 * j + 4 * lg + q;
          if (gn >= p.N) continue;
          float v = alpha * acc[i][j][q];
          if (R) v += ldf(R, (size_t)gm * p.ldr + gn);
          if (p.accumulate) v += ldf(C, (size_t)gm * p.ldc + gn);
          stf(C, (size_t)gm * p.ldc + gn, v);
        }
    }
  };

  u32x4_t fa0[GA], fa1[GA], fb0[TN], fb1[TN];
  {
    // ---- slabs of 64: THREE LDS units for one operand and TWO for the other (5 x 32 KiB = all of the 160 KiB) ----
    // The operand DMA of a slab has to land within one slab time when the ring is two deep on both sides, and
    // a burst of 64 KiB per CU takes about that long to deliver: the matrix pipes then wait for it every slab.
    // With a third unit, the "deep" operand is fetched one slab further ahead and only the other one's half of
    // the bytes is on the one-slab clock.  Slab kt lives in deep unit kt % 3 and shallow unit kt % 2; the barrier
    // of a slab sits before its last quarter.  Loads complete in order, so waiting for "all but the youngest
    // NDEEP" means everything older than the deep operand's youngest slab has landed.
#ifndef TIDE_RING_DEEPB
#define TIDE_RING_DEEPB 0
#endif
    constexpr bool DEEPB = TIDE_RING_DEEPB != 0;   // which operand owns the three units
    static_assert(A_STAGE == B_STAGE, "units are interchangeable");
    __shared__ __attribute__((aligned(1024))) bf16_t ld0[A_STAGE];
    __shared__ __attribute__((aligned(1024))) bf16_t ld1[A_STAGE];
    __shared__ __attribute__((aligned(1024))) bf16_t ld2[A_STAGE];
    __shared__ __attribute__((aligned(1024))) bf16_t ls0[B_STAGE];
    __shared__ __attribute__((aligned(1024))) bf16_t ls1[B_STAGE];
    auto deep = [&](auto U) -> bf16_t* {
      if constexpr (decltype(U)::value == 0) return ld0;
      else if constexpr (decltype(U)::value == 1) return ld1;
      else return ld2;
    };
    auto shal = [&](auto U) -> bf16_t* {
      if constexpr (decltype(U)::value == 0) return ls0;
      else return ls1;
    };
    auto unit_a = [&](auto D, auto S) -> bf16_t* { if constexpr (DEEPB) return shal(S); else return deep(D); };
    auto unit_b = [&](auto D, auto S) -> bf16_t* { if constexpr (DEEPB) return deep(D); else return shal(S); };
    typedef __attribute__((address_space(3))) bf16_t* lds_wp;
    auto lds_addr = [](bf16_t* q) -> uint32_t { return (uint32_t)(uintptr_t)(lds_wp)q; };
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    // The descriptor of an operand's next slab.  The loop asks for every slab of an operand once and in order, so
    // a running base address and a count of the k still to come are enough: a handful of scalar operations per
    // slab and no branch (computing pair, offset and extent from the slab number took twice as many, with
    // branches, in one burst between two quarters that the matrix pipes spent waiting).  When the count runs out
    // the walk moves on to the second operand pair, if there is one, and then to empty extents (the dummy slabs).
    // A K-major operand can be walked when every slab is whole; one with ragged K keeps the per-slab form
    // because its loads need k0 and K for their per-lane test.
    constexpr bool WALK_A = KWHOLE || AMM, WALK_B = KWHOLE || BNM;
    const int k_first = kt_lo * BK;                      // a split launch has one operand pair, so this is in pair 0
    const int k_span0 = min(p.K, (kt_lo + nk) * BK) - k_first;
    uint64_t a_base = (uint64_t)(a_tile0 + (AMM ? (size_t)k_first * p.lda : (size_t)k_first));
    uint64_t b_base = (uint64_t)(b_tile0 + (BNM ? (size_t)k_first * p.ldb : (size_t)k_first));
    uint64_t a_next = (uint64_t)a_tile1, b_next = (uint64_t)b_tile1;
    int a_rem = k_span0, b_rem = k_span0;
    int a_nrem = nkp2 > 0 ? p.K2 : 0, b_nrem = a_nrem;
    const uint32_t a_step = AMM ? (uint32_t)(2 * BK) * (uint32_t)p.lda : (uint32_t)(2 * BK);
    const uint32_t b_step = BNM ? (uint32_t)(2 * BK) * (uint32_t)p.ldb : (uint32_t)(2 * BK);
    // extent of a live slab: row-major over K: (rows of the slab - 1) * ld + columns left; K-major: (tile rows - 1) * ld + k left
    const uint32_t a_ext0 = AMM ? (uint32_t)(2 * (p.M - m0)) : (uint32_t)(2 * (a_rows - 1)) * (uint32_t)p.lda;
    const uint32_t b_ext0 = BNM ? (uint32_t)(2 * (p.N - n0)) : (uint32_t)(2 * (b_rows - 1)) * (uint32_t)p.ldb;
    auto walk = [&](auto RM, uint64_t& base, uint64_t& next, int& rem, int& nrem, uint32_t step, uint32_t ext0, int ld) {
      i32x4_t rs;
      const uint32_t bytes = decltype(RM)::value ? ext0 + (uint32_t)(min(rem, BK) - 1) * (uint32_t)(2 * ld) : ext0 + (uint32_t)(2 * rem);
      rs[0] = (int)(uint32_t)base; rs[1] = (int)((uint32_t)(base >> 32) & 0xffffu); rs[2] = rem > 0 ? (int)bytes : 0; rs[3] = 0x00020000;
      base += step;
      rem -= BK;
      const bool over = rem <= 0;
      base = over ? next : base;
      rem = over ? nrem : rem;
      nrem = over ? 0 : nrem;
      return rs;
    };
    auto desc_a = [&](int kt) {
      typename OpA::SlabDesc d;
      if constexpr (WALK_A) {
        d.k0 = 0; d.Kc = 0;
        d.rs = walk(std::bool_constant<AMM>{}, a_base, a_next, a_rem, a_nrem, a_step, a_ext0, p.lda);
      } else {
        int pr, k0, Kc;
        slab(kt, pr, k0, Kc);
        d = OpA::slab_desc(pr ? a_tile1 : a_tile0, p.lda, a_rows, p.M - m0, k0, Kc);
      }
      return d;
    };
    auto desc_b = [&](int kt) {
      typename OpB::SlabDesc d;
      if constexpr (WALK_B) {
        d.k0 = 0; d.Kc = 0;
        d.rs = walk(std::bool_constant<BNM>{}, b_base, b_next, b_rem, b_nrem, b_step, b_ext0, p.ldb);
      } else {
        int pr, k0, Kc;
        slab(kt, pr, k0, Kc);
        d = OpB::slab_desc(pr ? b_tile1 : b_tile0, p.ldb, b_rows, p.N - n0, k0, Kc);
      }
      return d;
    };
    auto dma_a = [&](auto I, const typename OpA::SlabDesc& d, bf16_t* unit) {
      if constexpr (WALK_A) OpA::template chunk_whole<decltype(I)::value>(d, lds_addr(unit), a_off, wave_s);
      else OpA::template chunk<decltype(I)::value>(d, lds_addr(unit), a_off, a_piece, wave_s);
    };
    auto dma_b = [&](auto I, const typename OpB::SlabDesc& d, bf16_t* unit) {
      if constexpr (WALK_B) OpB::template chunk_whole<decltype(I)::value>(d, lds_addr(unit), b_off, wave_s);
      else OpB::template chunk<decltype(I)::value>(d, lds_addr(unit), b_off, b_piece, wave_s);
    };
    constexpr int NDEEP = DEEPB ? NVB : NVA, NSHAL = DEEPB ? NVA : NVB;
    static_assert(GA + TN + NDEEP <= GA * TN && GA + TN + NSHAL <= GA * TN, "a quarter has a slot for every read and load it carries");
    auto desc_deep = [&](int kt) { if constexpr (DEEPB) return desc_b(kt); else return desc_a(kt); };
    auto desc_shal = [&](int kt) { if constexpr (DEEPB) return desc_a(kt); else return desc_b(kt); };
    auto dma_deep = [&](auto I, const auto& d, bf16_t* unit) { if constexpr (DEEPB) dma_b(I, d, unit); else dma_a(I, d, unit); };
    auto dma_shal = [&](auto I, const auto& d, bf16_t* unit) { if constexpr (DEEPB) dma_a(I, d, unit); else dma_b(I, d, unit); };
    auto all_deep = [&](bf16_t* unit, int kt) {
      const auto d = desc_deep(kt);
      [&]<int... I>(std::integer_sequence<int, I...>) { (dma_deep(Int<I>{}, d, unit), ...); }(std::make_integer_sequence<int, NDEEP>{});
    };
    auto all_shal = [&](bf16_t* unit, int kt) {
      const auto d = desc_shal(kt);
      [&]<int... I>(std::integer_sequence<int, I...>) { (dma_shal(Int<I>{}, d, unit), ...); }(std::make_integer_sequence<int, NSHAL>{});
    };
    // one fragment of A (index F of group G) / of B (index F) of the k32 step h of a unit
    auto frag_a = [&](const bf16_t* unit, int h, auto G, auto F, u32x4_t (&fa)[GA]) {
      u32x4_t t[1];
      OpA::template frags16<decltype(G)::value * GA + decltype(F)::value, 1>((lds_bf_t)unit, h, a_ro, t);
      fa[decltype(F)::value] = t[0];
    };
    auto frag_b = [&](const bf16_t* unit, int h, auto F, u32x4_t (&fb)[TN]) {
      u32x4_t t[1];
      OpB::template frags16<decltype(F)::value, 1>((lds_bf_t)unit, h, b_ro, t);
      fb[decltype(F)::value] = t[0];
    };
    // One quarter, instruction by instruction: MFMA X of A group G, then whatever `after(Int<X>)` issues (operand
    // reads of a later quarter, DMA loads); the order is pinned.
    auto quarter = [&](auto G, u32x4_t (&fa)[GA], u32x4_t (&fb)[TN], auto&& after) {
      constexpr int g0 = decltype(G)::value * GA;
      [&]<int... X>(std::integer_sequence<int, X...>) {
        ([&] {
          constexpr int i = X / TN, j = X % TN;
          acc[g0 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fb[j]),
                                                                   __builtin_bit_cast(bf16x8_t, fa[i]), acc[g0 + i][j], 0, 0, 0);
          after(Int<X>{});
          __builtin_amdgcn_sched_barrier(0);
        }(), ...);
      }(std::make_integer_sequence<int, NMF>{});
    };

    all_deep(ld0, 0);
    all_shal(ls0, 0);
    TIDE_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags_a(unit_a(Int<0>{}, Int<0>{}), 0, Int<0>{}, fa0);
    frags_b(unit_b(Int<0>{}, Int<0>{}), 0, fb0);
    all_deep(ld1, 1);
    all_shal(ls1, 1);
    __builtin_amdgcn_sched_barrier(0);
    // One slab: deep unit D, shallow unit S (fa0 / fb0 hold its first quarter's operands); the next slab's units
    // are DN, SN; DP is the deep unit the slab before vacated.
    auto step = [&](auto D, auto S, auto DN, auto SN, auto DP, int kt) {
      const bf16_t* ua = unit_a(D, S);
      const bf16_t* ubb = unit_b(D, S);
      quarter(Int<0>{}, fa0, fb0, [&](auto X) {
        if constexpr (decltype(X)::value < GA) frag_a(ua, 0, Int<1>{}, X, fa1);
      });
      const auto dd1 = desc_deep(kt + 2);
      quarter(Int<1>{}, fa1, fb0, [&](auto X) {
        constexpr int x = decltype(X)::value;
        if constexpr (x < GA) frag_a(ua, 1, Int<0>{}, X, fa0);
        else if constexpr (x < GA + TN) frag_b(ubb, 1, Int<x - GA>{}, fb1);
        else if constexpr (x < GA + TN + NDEEP) dma_deep(Int<x - GA - TN>{}, dd1, deep(DP));
      });
      quarter(Int<0>{}, fa0, fb1, [&](auto X) {
        if constexpr (decltype(X)::value < GA) frag_a(ua, 1, Int<1>{}, X, fa1);
      });
      // every operand read of this wave from the slab's units has returned; its share of the next slab (and of
      // everything older) has landed; only its youngest deep-operand loads may still be in flight
      __builtin_amdgcn_s_waitcnt((NDEEP & 15) | ((NDEEP >> 4) << 14));   // vmcnt(NDEEP), lgkmcnt(0), expcnt(0)
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      const bf16_t* uan = unit_a(DN, SN);
      const bf16_t* ubn = unit_b(DN, SN);
      const auto ds = desc_shal(kt + 2);
      quarter(Int<1>{}, fa1, fb1, [&](auto X) {
        constexpr int x = decltype(X)::value;
        if constexpr (x < GA) frag_a(uan, 0, Int<0>{}, X, fa0);
        else if constexpr (x < GA + TN) frag_b(ubn, 0, Int<x - GA>{}, fb0);
        // the shallow operand's loads follow the A reads (K-major B) or all eight reads (row-major B): measured,
        // 0.2-0.9 % per layout against issuing them beside the first reads
        constexpr int s0 = BNM ? GA + TN : GA;
        if constexpr (x >= s0 && x < s0 + NSHAL) dma_shal(Int<x - s0>{}, ds, shal(S));
      });
    };
    // The unit numbers repeat every six slabs.  The last round skips the slabs past nk one by one (a chain of
    // uniform branches with the single loop exit at the bottom: early exits out of the middle made the compiler
    // spill the accumulators).
    for (int kt = 0; kt < nk; kt += 6) {
      step(Int<0>{}, Int<0>{}, Int<1>{}, Int<1>{}, Int<2>{}, kt);
      if (__builtin_expect(kt + 1 < nk, 1)) step(Int<1>{}, Int<1>{}, Int<2>{}, Int<0>{}, Int<0>{}, kt + 1);
      if (__builtin_expect(kt + 2 < nk, 1)) step(Int<2>{}, Int<0>{}, Int<0>{}, Int<1>{}, Int<1>{}, kt + 2);
      if (__builtin_expect(kt + 3 < nk, 1)) step(Int<0>{}, Int<1>{}, Int<1>{}, Int<0>{}, Int<2>{}, kt + 3);
      if (__builtin_expect(kt + 4 < nk, 1)) step(Int<1>{}, Int<0>{}, Int<2>{}, Int<1>{}, Int<0>{}, kt + 4);
      if (__builtin_expect(kt + 5 < nk, 1)) step(Int<2>{}, Int<1>{}, Int<0>{}, Int<0>{}, Int<1>{}, kt + 5);
    }
    TIDE_WAIT_VMCNT(0);   // dummy slabs still in flight write LDS: let them land before the patches are written
    constexpr int PPU = A_STAGE / kPatchElems;   // epilogue patches per unit
    static_assert(PPU >= 1 && (NW + PPU - 1) / PPU <= 4, "the epilogue patches fit four units");
    const int pu = wave / PPU;
    bf16_t* unit = pu == 0 ? ld0 : (pu == 1 ? ld1 : (pu == 2 ? ld2 : ls0));
    epilogue(unit + (wave % PPU) * kPatchElems);
  }
}

// C[tile] += the partial sums of the later parts of every split tile, in the order of the parts (deterministic).
// Eight blocks per split tile (32 rows each); 256 threads, a thread adds 4 consecutive columns of 4 rows at a
// time, with the old values and every part's addends of those rows requested before the first sum.
__global__ __launch_bounds__(256) void splitk_fixup_kernel(float* __restrict__ C, int ldc, int M, int N, int tiles_n,
                                                           int split_full, int split_s, const float* __restrict__ scratch) {
  const int tiles_m = (M + 255) / 256;
  const int ntail = tiles_m * tiles_n - split_full;
  const int tile = blockIdx.x >> 3, rblk = blockIdx.x & 7;
  int tile_m, tile_n;
  tile_coords(split_full + tile, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * 256, n0 = tile_n * 256;
  const int c4 = (threadIdx.x & 63) * 4, r0 = rblk * 32 + (threadIdx.x >> 6);
  const int gn = n0 + c4;
  if (gn >= N) return;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    float4 v[4];
    bool ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = r0 + (half * 4 + i) * 4;
      ok[i] = m0 + r < M;
      v[i] = ok[i] ? *reinterpret_cast<const float4*>(C + (size_t)(m0 + r) * ldc + gn) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int j = 1; j < split_s; ++j) {
      float4 x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = r0 + (half * 4 + i) * 4;
        x[i] = *reinterpret_cast<const float4*>(scratch + ((size_t)(j - 1) * ntail + tile) * 65536 + (size_t)r * 256 + c4);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) { v[i].x += x[i].x; v[i].y += x[i].y; v[i].z += x[i].z; v[i].w += x[i].w; }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = r0 + (half * 4 + i) * 4;
      if (ok[i]) *reinterpret_cast<float4*>(C + (size_t)(m0 + r) * ldc + gn) = v[i];
    }
  }
}

namespace {
// How the last round of a 256 x 256-tile launch is split over K: fp32 results without residual on tiles that do
// not fill the last round of the 256 CUs (at most half of it: otherwise two parts per tile would not fit the round).
struct SplitPlan { int s, full; size_t bytes; };
SplitPlan plan_split(const GemmArgs& a) {
  SplitPlan sp{1, 0, 0};
#ifdef TIDE_NO_SPLITK
  return sp;
#endif
  if (a.out_dtype != kF32 || a.residual || a.A2 || a.m_dev) return sp;
  if ((a.ldc % 4) || (a.N % 4) || (((uintptr_t)a.C) & 15)) return sp;
  const int64_t tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (tiles < 200) return sp;
  const int rem = (int)(tiles % 256);
  if (rem == 0 || rem > 128) return sp;
  const int64_t slabs = (a.K + 31) / 32;
  int s = 256 / rem;
  if (s > 8) s = 8;
  while (s > 1 && slabs / s < 32) --s;       // a part keeps at least 32 slabs (1024 k): below that its fixed cost dominates
  if (s <= 1) return sp;
  sp.s = s; sp.full = (int)(tiles - rem);
  sp.bytes = (size_t)(s - 1) * (size_t)rem * 65536 * sizeof(float);
  return sp;
}
}  // namespace

size_t gemm_splitk_scratch_bytes(const GemmArgs& a) { return gemm_mfma_supported(a) ? plan_split(a).bytes : 0; }

bool gemm_mfma_supported(const GemmArgs& a) {
  if (a.in_dtype != kBF16) return false;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
  if (a.lda % 8 || a.ldb % 8 || a.K % 8) return false;
  if (a.A2 && (a.K2 <= 0 || a.K2 % 8 || !a.B2 || a.k_dev)) return false;
  if (((uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.A2 | (uintptr_t)a.B2) & 15) return false;
  // 32-bit byte offsets inside one tile
  const int64_t lim = (int64_t)1 << 21;
  if (a.lda >= lim || a.ldb >= lim || a.ldc >= lim) return false;
  if (a.M >= ((int64_t)1 << 24) || a.N >= ((int64_t)1 << 24) || a.K >= ((int64_t)1 << 24) || a.K2 >= ((int64_t)1 << 24)) return false;
  if (a.layout == kNN || a.layout == kTN) {
    if (a.N % 8) return false;  // B rows are read in 16-byte pieces along N
  }
  if (a.layout == kTN && a.M % 8) return false;
  return true;
}

namespace {

template <int BM, int BN, int NW, bool AMM, bool BNM, typename TO, int BK>
hipError_t launch_cfg(const MfmaParams& p, hipStream_t s) {
  MfmaParams q = p;
  q.tiles_m = (p.M + BM - 1) / BM;
  q.tiles_n = (p.N + BN - 1) / BN;
  hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, NW, AMM, BNM, TO, BK>), dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(NW * 64), 0,
                     s, q);
  return hipGetLastError();
}

bool use_big_tiles(int64_t M, int64_t N) { return ((M + 255) / 256) * ((N + 255) / 256) >= 200; }

template <bool AMM, bool BNM, typename TO>
hipError_t launch_layout(const MfmaParams& p, hipStream_t s) {
  // slab depth of the 32x32x16 kernels: 64 (two stages) as soon as one operand is K-major, else 32 (four stages);
  // the 16x16x32 kernel walks slabs of 64 in every layout
  constexpr int BK = (AMM && BNM) ? 32 : 64;
#ifndef TIDE_BIG_TILE_MFMA32
  if (use_big_tiles(p.M, p.N)) {
    MfmaParams q = p;
    q.tiles_m = (p.M + 255) / 256;
    q.tiles_n = (p.N + 255) / 256;
    const int tiles = q.tiles_m * q.tiles_n;
    const int items = q.split_s > 1 ? q.split_full + (tiles - q.split_full) * q.split_s : tiles;
#ifndef TIDE_GEMM_WAVES_N
#define TIDE_GEMM_WAVES_N 4
#endif
    constexpr int WAVES_N = TIDE_GEMM_WAVES_N;
    // every slab whole (and K known on the host): the DMA loads of a K-major operand take loop-constant lane offsets
    // (with both operands row-major over K the two forms are the same code: one instantiation)
    const bool whole = !(AMM && BNM) && !p.k_dev && p.K % 64 == 0 && (!p.A2 || p.K2 % 64 == 0);
    if (whole) hipLaunchKernelGGL((gemm_mfma16_kernel<AMM, BNM, TO, 64, WAVES_N, true>), dim3((unsigned)items), dim3(2 * WAVES_N * 64), 0, s, q);
    else hipLaunchKernelGGL((gemm_mfma16_kernel<AMM, BNM, TO, 64, WAVES_N, false>), dim3((unsigned)items), dim3(2 * WAVES_N * 64), 0, s, q);
    return hipGetLastError();
  }
#endif
  if (p.split_s > 1) return hipErrorInvalidValue;   // only the 16x16x32 kernel knows the split
  if (use_big_tiles(p.M, p.N)) return launch_cfg<256, 256, 8, AMM, BNM, TO, BK>(p, s);
  return launch_cfg<128, 128, 4, AMM, BNM, TO, BK>(p, s);
}

const char* gemm_kernel_name(const GemmArgs& a) {
  if (!gemm_mfma_supported(a)) return "gemm_simple";
  const bool big = use_big_tiles(a.M, a.N);
  const bool f32 = a.out_dtype == kF32;
  switch (a.layout) {
    case kNT: return big ? (f32 ? "gemm_mfma_nt_256_f32out" : "gemm_mfma_nt_256_bf16out") : (f32 ? "gemm_mfma_nt_128_f32out" : "gemm_mfma_nt_128_bf16out");
    case kNN: return big ? (f32 ? "gemm_mfma_nn_256_f32out" : "gemm_mfma_nn_256_bf16out") : (f32 ? "gemm_mfma_nn_128_f32out" : "gemm_mfma_nn_128_bf16out");
    default: return big ? (f32 ? "gemm_mfma_tn_256_f32out" : "gemm_mfma_tn_256_bf16out") : (f32 ? "gemm_mfma_tn_128_f32out" : "gemm_mfma_tn_128_bf16out");
  }
}

}  // namespace

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s) {
  MfmaParams p;
  p.A = (const bf16_t*)a.A; p.B = (const bf16_t*)a.B;
  p.A2 = (const bf16_t*)a.A2; p.B2 = (const bf16_t*)a.B2;
  p.C = a.C; p.R = a.residual; p.alpha_dev = a.alpha_dev;
  p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K; p.K2 = a.A2 ? (int)a.K2 : 0;
  p.lda = (int)a.lda; p.ldb = (int)a.ldb; p.ldc = (int)a.ldc; p.ldr = (int)a.ldr;
  p.alpha = a.alpha; p.accumulate = a.accumulate; p.tiles_m = p.tiles_n = 0;
  p.m_dev = a.m_dev; p.m_off = (int)a.m_off; p.k_dev = a.k_dev; p.k_off = (int)a.k_off;
  p.split_s = 1; p.split_full = 0; p.split_scratch = nullptr;
  const SplitPlan sp = plan_split(a);
  if (sp.s > 1 && a.scratch && a.scratch_bytes >= sp.bytes && (((uintptr_t)a.scratch) & 15) == 0) {
    p.split_s = sp.s; p.split_full = sp.full; p.split_scratch = (float*)a.scratch;
  }
  const bool f32out = a.out_dtype == kF32;
  hipError_t e = hipErrorInvalidValue;
  switch (a.layout) {
    case kNT: e = f32out ? launch_layout<false, false, float>(p, s) : launch_layout<false, false, bf16_t>(p, s); break;
    case kNN: e = f32out ? launch_layout<false, true, float>(p, s) : launch_layout<false, true, bf16_t>(p, s); break;
    case kTN: e = f32out ? launch_layout<true, true, float>(p, s) : launch_layout<true, true, bf16_t>(p, s); break;
  }
  if (e != hipSuccess || p.split_s <= 1) return e;
  const int tiles_n = (p.N + 255) / 256;
  const int ntail = ((p.M + 255) / 256) * tiles_n - p.split_full;
  hipLaunchKernelGGL(splitk_fixup_kernel, dim3((unsigned)ntail * 8u), dim3(256), 0, s, (float*)p.C, p.ldc, p.M, p.N, tiles_n,
                     p.split_full, p.split_s, p.split_scratch);
  return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  // algorithmic work of the call, for the optional profiler
  const double k = (double)a.K + (a.A2 ? (double)a.K2 : 0.0);
  const double es_in = (double)dtype_size(a.in_dtype), es_out = (double)dtype_size(a.out_dtype);
  const double bytes = es_in * k * ((double)a.M + (double)a.N) +
                       es_out * (double)a.M * (double)a.N * (1.0 + (a.accumulate ? 1.0 : 0.0) + (a.residual ? 1.0 : 0.0));
  ProfScope ps(gemm_kernel_name(a), 2.0 * (double)a.M * (double)a.N * k, bytes, s);
  if (a.m_dev) prof_dynamic(a.m_dev, a.m_off, a.M);
  else if (a.k_dev) prof_dynamic(a.k_dev, a.k_off, a.K);
  if (gemm_mfma_supported(a)) return launch_gemm_mfma(a, s);
  return launch_gemm_simple(a, s);
}

// ------------------------------------------------------------------------------------------------
// Pure-MFMA probe: what the matrix pipes deliver with nothing else going on (operands in registers, no
// LDS, no memory).  8 waves per block, 8 independent accumulators per wave.  The operands are random bf16 values
// (random sign and mantissa, magnitude in [0.5, 2)), a different pair for each of the 8 MFMAs: what the pipes draw
// depends on how many operand bits change from one instruction to the next, and under its package power limit the
// chip sustains 1.84 PFLOP/s on such operands against 2.45 PFLOP/s on constant ones.  Timed over a few hundred
// milliseconds, the rate is the practical ceiling for the GEMM above.
// ------------------------------------------------------------------------------------------------
namespace {
__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
__device__ __forceinline__ uint32_t probe_pair(uint32_t seed) {   // two bf16 values with |x| in [0.5, 2)
  const uint32_t h = probe_hash(seed);
  const uint32_t lo = 0x3F00u | (h & 0x80FFu) | ((h >> 9) & 0x0080u);
  const uint32_t hi = 0x3F00u | ((h >> 16) & 0x80FFu) | ((h >> 3) & 0x0080u);
  return lo | (hi << 16);
}
}  // namespace

__global__ __launch_bounds__(512) void mfma_probe_kernel(float* __restrict__ sink, int iters) {
  const uint32_t tid = blockIdx.x * 512u + threadIdx.x;
  u32x4_t a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      a[j][w] = probe_pair(tid * 64u + j * 4 + w);
      b[j][w] = probe_pair(tid * 64u + 32 + j * 4 + w);
    }
  f32x16_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[j]), __builtin_bit_cast(bf16x8_t, b[(j + 3) & 7]), acc[j], 0, 0, 0);
  }
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) v += acc[j][q];
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = v;
}

hipError_t launch_mfma_probe(int blocks, int iters, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3(512), 0, s, sink, iters);
  return hipGetLastError();
}

}  // namespace tide

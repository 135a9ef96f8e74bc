// bf16 MFMA GEMM for gfx950 (CDNA4), fp32 accumulation, for the three layouts of the training step:
//   NT  C = A[M,K] B[N,K]^T   forward projections           (both operands K-contiguous)
//   NN  C = A[M,K] B[K,N]     input gradients dX = dY W     (B is N-contiguous)
//   TN  C = A[K,M]^T B[K,N]   weight gradients dW = dY^T X  (both operands contracted over rows)
//
// Design
//   * One 256-thread block (4 wavefronts, 2x2) computes a BM x BN tile (256x256 or 128x128) with
//     v_mfma_f32_32x32x16_bf16; each wave owns a (BM/2)x(BN/2) sub-tile = TMxTN MFMA tiles.
//   * K is walked in slabs of 64.  Slabs go global -> registers (buffer loads, 16 B per lane, hardware
//     zero-fill outside the tile's valid extent, so ragged M/N/K need no special code) -> LDS, double
//     buffered: the loads of slab k+1 are in flight while the MFMAs of slab k run.
//   * An operand whose contraction index is contiguous in memory ("K-major") is kept as [row][k] in LDS
//     (row pitch 64+8 elements: conflict-free 16-byte reads) and fetched as one 16-byte read per MFMA
//     operand.  An operand whose contraction index is the slow one ("row-major over K", the B of NN and
//     both operands of TN) is kept exactly as in memory, [k][row], and transposed on the way to the
//     MFMA: each lane reads TM consecutive rows for 8 consecutive k (8 narrow LDS reads) and regroups
//     the 16-bit halves with v_perm_b32.  The MFMA tile i of a wave then covers rows {TM*r + i}, an
//     interleaving the epilogue undoes.  No transposed copy of any operand is ever written to HBM.
//   * The contraction may run over two operand pairs back to back (used for
//     d b = dGate W_gate + dUp W_up), and the epilogue fuses alpha (host and device scalar), a
//     residual add, accumulation into C, and the output cast.
//   * Work-groups are renumbered so that each of the 8 XCDs (round-robin dispatch) gets a contiguous
//     range of tiles, walked in groups of 8 tile-rows, which keeps the A/B panels of neighbouring tiles
//     in that XCD's L2.
#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr int KPAD = 8;  // LDS row padding in elements (16 bytes)

struct MfmaParams {
  const bf16_t* A; const bf16_t* B; const bf16_t* A2; const bf16_t* B2;
  void* C; const void* R; const float* alpha_dev;
  int M, N, K, K2;
  int lda, ldb, ldc, ldr;
  float alpha;
  int accumulate;
  int tiles_m, tiles_n;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

template <int BM, int BN, bool AMM, bool BNM, typename TO>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(MfmaParams p) {
  constexpr int WM = BM / 2, WN = BN / 2;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_PITCH = AMM ? (BM + KPAD) : (BK + KPAD);
  constexpr int B_PITCH = BNM ? (BN + KPAD) : (BK + KPAD);
  constexpr int A_STAGE = AMM ? BK * A_PITCH : BM * A_PITCH;  // elements
  constexpr int B_STAGE = BNM ? BK * B_PITCH : BN * B_PITCH;
  constexpr int NLA = BM * BK / 8 / 256;  // 16-byte pieces per thread per slab
  constexpr int NLB = BN * BK / 8 / 256;

  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* sA = smem;                 // [2][A_STAGE]
  bf16_t* sB = smem + 2 * A_STAGE;   // [2][B_STAGE]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int lr = lane & 31, lg = lane >> 5;

  // ---- XCD-aware tile numbering ----
  int tile_m, tile_n;
  {
    const int nb = p.tiles_m * p.tiles_n;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, idx = pid >> 3;
    const int q = nb >> 3, r = nb & 7;
    const int v = xcd * q + min(xcd, r) + idx;  // contiguous range per XCD
    constexpr int GROUP = 8;
    const int per_group = GROUP * p.tiles_n;
    const int gid = v / per_group;
    const int first_m = gid * GROUP;
    const int gsz = min(p.tiles_m - first_m, GROUP);
    const int in_g = v - gid * per_group;
    tile_m = first_m + in_g % gsz;
    tile_n = in_g / gsz;
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  const int nk1 = (p.K + BK - 1) / BK;
  const int nk2 = p.A2 ? (p.K2 + BK - 1) / BK : 0;
  const int nk = nk1 + nk2;

  i32x4_t ra[NLA], rb[NLB];

  // global -> registers for slab kt
  auto gload = [&](int kt) {
    const bool second = kt >= nk1;
    const bf16_t* Ab = second ? p.A2 : p.A;
    const bf16_t* Bb = second ? p.B2 : p.B;
    const int Kc = second ? p.K2 : p.K;
    const int k0 = (second ? kt - nk1 : kt) * BK;
    if (AMM) {
      constexpr int PPR = BM / 8;        // pieces per k-row
      constexpr int RSTEP = 256 / PPR;   // k-rows covered per pass
      const int rows_valid = min(BK, Kc - k0);
      const bf16_t* base = Ab + (size_t)k0 * p.lda + m0;
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (uint32_t)(((int64_t)(rows_valid - 1) * p.lda + (p.M - m0)) * 2));
      const int piece = tid % PPR, kr = tid / PPR;
#pragma unroll
      for (int i = 0; i < NLA; ++i)
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (uint32_t)(((kr + i * RSTEP) * p.lda + piece * 8) * 2), 0, 0);
    } else {
      const int rows_valid = min(BM, p.M - m0);
      const bf16_t* base = Ab + (size_t)m0 * p.lda;
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (uint32_t)(((int64_t)(rows_valid - 1) * p.lda + Kc) * 2));
      const int piece = tid & 7, row = tid >> 3;
      const int kc = k0 + piece * 8;
#pragma unroll
      for (int i = 0; i < NLA; ++i) {
        uint32_t off = (uint32_t)(((row + i * 32) * p.lda + kc) * 2);
        if (kc >= Kc) off = 0x7FFFFFF0u;
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
      }
    }
    if (BNM) {
      constexpr int PPR = BN / 8;
      constexpr int RSTEP = 256 / PPR;
      const int rows_valid = min(BK, Kc - k0);
      const bf16_t* base = Bb + (size_t)k0 * p.ldb + n0;
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (uint32_t)(((int64_t)(rows_valid - 1) * p.ldb + (p.N - n0)) * 2));
      const int piece = tid % PPR, kr = tid / PPR;
#pragma unroll
      for (int i = 0; i < NLB; ++i)
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, (uint32_t)(((kr + i * RSTEP) * p.ldb + piece * 8) * 2), 0, 0);
    } else {
      const int rows_valid = min(BN, p.N - n0);
      const bf16_t* base = Bb + (size_t)n0 * p.ldb;
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (uint32_t)(((int64_t)(rows_valid - 1) * p.ldb + Kc) * 2));
      const int piece = tid & 7, row = tid >> 3;
      const int kc = k0 + piece * 8;
#pragma unroll
      for (int i = 0; i < NLB; ++i) {
        uint32_t off = (uint32_t)(((row + i * 32) * p.ldb + kc) * 2);
        if (kc >= Kc) off = 0x7FFFFFF0u;
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
      }
    }
  };

  // registers -> LDS stage st
  auto sstore = [&](int st) {
    bf16_t* a = sA + st * A_STAGE;
    bf16_t* b = sB + st * B_STAGE;
    if (AMM) {
      constexpr int PPR = BM / 8;
      constexpr int RSTEP = 256 / PPR;
      const int piece = tid % PPR, kr = tid / PPR;
#pragma unroll
      for (int i = 0; i < NLA; ++i)
        *reinterpret_cast<i32x4_t*>(a + (kr + i * RSTEP) * A_PITCH + piece * 8) = ra[i];
    } else {
      const int piece = tid & 7, row = tid >> 3;
#pragma unroll
      for (int i = 0; i < NLA; ++i)
        *reinterpret_cast<i32x4_t*>(a + (row + i * 32) * A_PITCH + piece * 8) = ra[i];
    }
    if (BNM) {
      constexpr int PPR = BN / 8;
      constexpr int RSTEP = 256 / PPR;
      const int piece = tid % PPR, kr = tid / PPR;
#pragma unroll
      for (int i = 0; i < NLB; ++i)
        *reinterpret_cast<i32x4_t*>(b + (kr + i * RSTEP) * B_PITCH + piece * 8) = rb[i];
    } else {
      const int piece = tid & 7, row = tid >> 3;
#pragma unroll
      for (int i = 0; i < NLB; ++i)
        *reinterpret_cast<i32x4_t*>(b + (row + i * 32) * B_PITCH + piece * 8) = rb[i];
    }
  };

  // LDS -> MFMA operand fragments for k16 step kk of stage st
  auto frag_load = [&](int st, int kk, u32x4_t (&fa)[TM], u32x4_t (&fb)[TN]) {
    const bf16_t* a = sA + st * A_STAGE;
    const bf16_t* b = sB + st * B_STAGE;
    if (AMM) {
      const bf16_t* src = a + (kk * 16 + lg * 8) * A_PITCH + wave_m * WM + TM * lr;
      if (TM == 4) {
        uint2 r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const uint2*>(src + j * A_PITCH);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t lo = (i < 2) ? r[2 * w].x : r[2 * w].y;
            const uint32_t hi = (i < 2) ? r[2 * w + 1].x : r[2 * w + 1].y;
            fa[i][w] = __builtin_amdgcn_perm(hi, lo, (i & 1) ? 0x07060302u : 0x05040100u);
          }
      } else {
        uint32_t r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const uint32_t*>(src + j * A_PITCH);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int w = 0; w < 4; ++w)
            fa[i][w] = __builtin_amdgcn_perm(r[2 * w + 1], r[2 * w], (i & 1) ? 0x07060302u : 0x05040100u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const u32x4_t*>(a + (wave_m * WM + 32 * i + lr) * A_PITCH + kk * 16 + lg * 8);
    }
    if (BNM) {
      const bf16_t* src = b + (kk * 16 + lg * 8) * B_PITCH + wave_n * WN + TN * lr;
      if (TN == 4) {
        uint2 r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const uint2*>(src + j * B_PITCH);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t lo = (i < 2) ? r[2 * w].x : r[2 * w].y;
            const uint32_t hi = (i < 2) ? r[2 * w + 1].x : r[2 * w + 1].y;
            fb[i][w] = __builtin_amdgcn_perm(hi, lo, (i & 1) ? 0x07060302u : 0x05040100u);
          }
      } else {
        uint32_t r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const uint32_t*>(src + j * B_PITCH);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int w = 0; w < 4; ++w)
            fb[i][w] = __builtin_amdgcn_perm(r[2 * w + 1], r[2 * w], (i & 1) ? 0x07060302u : 0x05040100u);
      }
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const u32x4_t*>(b + (wave_n * WN + 32 * j + lr) * B_PITCH + kk * 16 + lg * 8);
    }
  };

  if (nk > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    u32x4_t fa[2][TM], fb[2][TN];
    frag_load(st, 0, fa[0], fb[0]);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) frag_load(st, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
      // keep the operand reads of step kk+1 ahead of the MFMAs of step kk (the scheduler would
      // otherwise sink each read next to its first use and expose the LDS latency)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8_t, fa[kk & 1][i]), __builtin_bit_cast(bf16x8_t, fb[kk & 1][j]),
              acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kt + 1 < nk) sstore(st ^ 1);
    __syncthreads();
  }

  // ---- epilogue ----
  float alpha = p.alpha;
  if (p.alpha_dev) alpha *= *p.alpha_dev;
  TO* C = (TO*)p.C;
  const TO* R = (const TO*)p.R;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int rr = 8 * (q >> 2) + 4 * lg + (q & 3);
      const int gm = m0 + wave_m * WM + (AMM ? (TM * rr + i) : (32 * i + rr));
      if (gm >= p.M) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int gn = n0 + wave_n * WN + (BNM ? (TN * lr + j) : (32 * j + lr));
        if (gn >= p.N) continue;
        float v = alpha * acc[i][j][q];
        if (R) v += ldf(R, (size_t)gm * p.ldr + gn);
        if (p.accumulate) v += ldf(C, (size_t)gm * p.ldc + gn);
        stf(C, (size_t)gm * p.ldc + gn, v);
      }
    }
  }
}

bool gemm_mfma_supported(const GemmArgs& a) {
  if (a.in_dtype != kBF16) return false;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
  if (a.lda % 8 || a.ldb % 8 || a.K % 8) return false;
  if (a.A2 && (a.K2 <= 0 || a.K2 % 8 || !a.B2)) return false;
  if (((uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.A2 | (uintptr_t)a.B2) & 15) return false;
  // 32-bit byte offsets inside one tile
  const int64_t lim = (int64_t)1 << 21;
  if (a.lda >= lim || a.ldb >= lim || a.ldc >= lim) return false;
  if (a.M >= ((int64_t)1 << 24) || a.N >= ((int64_t)1 << 24) || a.K >= ((int64_t)1 << 24)) return false;
  if (a.layout == kNN || a.layout == kTN) {
    if (a.N % 8) return false;  // B rows are read in 16-byte pieces along N
  }
  if (a.layout == kTN && a.M % 8) return false;
  return true;
}

template <int BM, int BN, bool AMM, bool BNM, typename TO>
static hipError_t launch_cfg(const MfmaParams& p, hipStream_t s) {
  constexpr int A_PITCH = AMM ? (BM + KPAD) : (BK + KPAD);
  constexpr int B_PITCH = BNM ? (BN + KPAD) : (BK + KPAD);
  constexpr int A_STAGE = AMM ? BK * A_PITCH : BM * A_PITCH;
  constexpr int B_STAGE = BNM ? BK * B_PITCH : BN * B_PITCH;
  constexpr size_t smem = (size_t)2 * (A_STAGE + B_STAGE) * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<BM, BN, AMM, BNM, TO>;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  MfmaParams q = p;
  q.tiles_m = (p.M + BM - 1) / BM;
  q.tiles_n = (p.N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(256), smem, s, q);
  return hipGetLastError();
}

template <bool AMM, bool BNM, typename TO>
static hipError_t launch_layout(const MfmaParams& p, hipStream_t s) {
  const int64_t big_tiles = (int64_t)((p.M + 255) / 256) * ((p.N + 255) / 256);
  if (big_tiles >= 200) return launch_cfg<256, 256, AMM, BNM, TO>(p, s);
  return launch_cfg<128, 128, AMM, BNM, TO>(p, s);
}

hipError_t launch_gemm_mfma(const GemmArgs& a, hipStream_t s) {
  MfmaParams p;
  p.A = (const bf16_t*)a.A; p.B = (const bf16_t*)a.B;
  p.A2 = (const bf16_t*)a.A2; p.B2 = (const bf16_t*)a.B2;
  p.C = a.C; p.R = a.residual; p.alpha_dev = a.alpha_dev;
  p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K; p.K2 = a.A2 ? (int)a.K2 : 0;
  p.lda = (int)a.lda; p.ldb = (int)a.ldb; p.ldc = (int)a.ldc; p.ldr = (int)a.ldr;
  p.alpha = a.alpha; p.accumulate = a.accumulate; p.tiles_m = p.tiles_n = 0;
  const bool f32out = a.out_dtype == kF32;
  switch (a.layout) {
    case kNT: return f32out ? launch_layout<false, false, float>(p, s) : launch_layout<false, false, bf16_t>(p, s);
    case kNN: return f32out ? launch_layout<false, true, float>(p, s) : launch_layout<false, true, bf16_t>(p, s);
    case kTN: return f32out ? launch_layout<true, true, float>(p, s) : launch_layout<true, true, bf16_t>(p, s);
  }
  return hipErrorInvalidValue;
}

static const char* gemm_kernel_name(const GemmArgs& a) {
  if (!gemm_mfma_supported(a)) return "gemm_simple";
  const bool big = ((a.M + 255) / 256) * ((a.N + 255) / 256) >= 200;
  const bool f32 = a.out_dtype == kF32;
  switch (a.layout) {
    case kNT: return big ? (f32 ? "gemm_mfma_nt_256_f32out" : "gemm_mfma_nt_256_bf16out") : (f32 ? "gemm_mfma_nt_128_f32out" : "gemm_mfma_nt_128_bf16out");
    case kNN: return big ? (f32 ? "gemm_mfma_nn_256_f32out" : "gemm_mfma_nn_256_bf16out") : (f32 ? "gemm_mfma_nn_128_f32out" : "gemm_mfma_nn_128_bf16out");
    default: return big ? (f32 ? "gemm_mfma_tn_256_f32out" : "gemm_mfma_tn_256_bf16out") : (f32 ? "gemm_mfma_tn_128_f32out" : "gemm_mfma_tn_128_bf16out");
  }
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  // algorithmic work of the call, for the optional profiler
  const double k = (double)a.K + (a.A2 ? (double)a.K2 : 0.0);
  const double es_in = (double)dtype_size(a.in_dtype), es_out = (double)dtype_size(a.out_dtype);
  const double bytes = es_in * k * ((double)a.M + (double)a.N) +
                       es_out * (double)a.M * (double)a.N * (1.0 + (a.accumulate ? 1.0 : 0.0) + (a.residual ? 1.0 : 0.0));
  ProfScope ps(gemm_kernel_name(a), 2.0 * (double)a.M * (double)a.N * k, bytes, s);
  if (gemm_mfma_supported(a)) return launch_gemm_mfma(a, s);
  return launch_gemm_simple(a, s);
}

}  // namespace tide

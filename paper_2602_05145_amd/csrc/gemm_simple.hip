// Shape-agnostic GEMM for gfx950: any sizes, strides and dtype (fp32 or bf16 storage, fp32 FMA
// arithmetic).  It is the whole GEMM path of fp32 mode (where the step is latency-bound and exactness
// matters) and the fallback of bf16 mode for shapes the MFMA kernel does not take (unaligned leading
// dimensions).  64x64 output tile per 256-thread block, 4x4 micro-tile per thread, LDS-staged K slabs.
#include "kernels.h"
#include "tide_common.h"

namespace tide {

struct SimpleGemmParams {
  const void* A; const void* B; const void* A2; const void* B2;
  void* C; const void* R; const float* alpha_dev;
  int64_t M, N, K, K2;
  int64_t sam, sak, sbn, sbk, ldc, ldr;
  float alpha;
  int accumulate;
  const int* m_dev; int64_t m_off;
  const int* k_dev; int64_t k_off;
};

template <typename TI, typename TO>
__global__ __launch_bounds__(256) void gemm_simple_kernel(SimpleGemmParams p) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
  // sizes that are only known on the device (block-uniform)
  if (p.m_dev) p.M = max((int64_t)0, min(p.M, (int64_t)*p.m_dev - p.m_off));
  if (p.k_dev) p.K = max((int64_t)0, min(p.K, (int64_t)*p.k_dev - p.k_off));
  if (m0 >= p.M) return;
  if (p.K == 0 && p.K2 == 0 && p.accumulate) return;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int pair = 0; pair < 2; ++pair) {
    const TI* A = (const TI*)(pair ? p.A2 : p.A);
    const TI* B = (const TI*)(pair ? p.B2 : p.B);
    const int64_t K = pair ? p.K2 : p.K;
    if (A == nullptr || K <= 0) continue;
    for (int64_t k0 = 0; k0 < K; k0 += BK) {
      // 64x16 elements per operand, 4 per thread
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int idx = threadIdx.x + e * 256;
        // consecutive threads walk the contiguous dimension of each operand
        int am, ak;
        if (p.sak == 1) { ak = idx & 15; am = idx >> 4; } else { am = idx & 63; ak = idx >> 6; }
        const int64_t gm = m0 + am, gk = k0 + ak;
        As[ak][am] = (gm < p.M && gk < K) ? ldf(A, (size_t)(gm * p.sam + gk * p.sak)) : 0.f;
        int bn, bk;
        if (p.sbk == 1) { bk = idx & 15; bn = idx >> 4; } else { bn = idx & 63; bk = idx >> 6; }
        const int64_t gn = n0 + bn, gk2 = k0 + bk;
        Bs[bk][bn] = (gn < p.N && gk2 < K) ? ldf(B, (size_t)(gn * p.sbn + gk2 * p.sbk)) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
  float alpha = p.alpha;
  if (p.alpha_dev) alpha *= *p.alpha_dev;
  TO* C = (TO*)p.C;
  const TO* R = (const TO*)p.R;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t gm = m0 + ty * 4 + i;
    if (gm >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t gn = n0 + tx * 4 + j;
      if (gn >= p.N) continue;
      float v = alpha * acc[i][j];
      if (R) v += ldf(R, (size_t)(gm * p.ldr + gn));
      if (p.accumulate) v += ldf(C, (size_t)(gm * p.ldc + gn));
      stf(C, (size_t)(gm * p.ldc + gn), v);
    }
  }
}

hipError_t launch_gemm_simple(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  SimpleGemmParams p;
  p.A = a.A; p.B = a.B; p.A2 = a.A2; p.B2 = a.B2; p.C = a.C; p.R = a.residual; p.alpha_dev = a.alpha_dev;
  p.M = a.M; p.N = a.N; p.K = a.K; p.K2 = a.A2 ? a.K2 : 0;
  p.ldc = a.ldc; p.ldr = a.ldr; p.alpha = a.alpha; p.accumulate = a.accumulate;
  p.m_dev = a.m_dev; p.m_off = a.m_off; p.k_dev = a.k_dev; p.k_off = a.k_off;
  switch (a.layout) {
    case kNT: p.sam = a.lda; p.sak = 1; p.sbn = a.ldb; p.sbk = 1; break;
    case kNN: p.sam = a.lda; p.sak = 1; p.sbn = 1; p.sbk = a.ldb; break;
    case kTN: p.sam = 1; p.sak = a.lda; p.sbn = 1; p.sbk = a.ldb; break;
    default: return hipErrorInvalidValue;
  }
  dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64)), blk(256);
  if (grid.y > 65535) return hipErrorInvalidValue;
  if (a.in_dtype == kBF16 && a.out_dtype == kBF16) hipLaunchKernelGGL((gemm_simple_kernel<bf16_t, bf16_t>), grid, blk, 0, s, p);
  else if (a.in_dtype == kBF16 && a.out_dtype == kF32) hipLaunchKernelGGL((gemm_simple_kernel<bf16_t, float>), grid, blk, 0, s, p);
  else if (a.in_dtype == kF32 && a.out_dtype == kF32) hipLaunchKernelGGL((gemm_simple_kernel<float, float>), grid, blk, 0, s, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace tide

// Shape-agnostic causal grouped-query attention for gfx950: one wavefront per query row (forward, dQ)
// or per key row (dK, dV), fp32 arithmetic, any head_dim <= 256 and any sequence length.  It is the
// attention path of fp32 mode and the bf16 fallback for head sizes the MFMA kernel does not take.
// Deterministic: no atomics; every output element is produced by exactly one wave in a fixed order.
//
// Activation layout: qkv [B*S, (nh + 2 nkv) dh] with q heads first, then k heads, then v heads; query
// head h reads kv head h / (nh / nkv).  lse[b, h, i] is the log-sum-exp of the scaled scores of row i.
// Packed batches (cu_seqlens given): sequence b owns rows [cu[b], cu[b+1]) and lse / delta are [nh, T].
#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

constexpr int kMaxDh = 256;
constexpr int kDhSlots = kMaxDh / 64;

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_simple_kernel(const T* __restrict__ qkv, T* __restrict__ out,
                                                             float* __restrict__ lse, int Smax, int nh, int nkv,
                                                             int dh, const int* __restrict__ cu, int64_t Trows) {
  __shared__ float qs[kMaxDh];
  __shared__ float ps[64];
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const SeqView sv = seq_view(cu, b, Smax, Trows);
  if (i >= sv.len) return;   // whole block: the sequence is shorter than the grid
  const size_t row0 = (size_t)sv.row0;
  const int lane = threadIdx.x;
  const int G = nh / nkv, kh = h / G;
  const int ld = (nh + 2 * nkv) * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t rowq = (row0 + i) * ld;
  for (int c = lane; c < dh; c += 64) qs[c] = ldf(qkv, rowq + (size_t)h * dh + c) * scale;
  __syncthreads();
  const size_t koff = (size_t)(nh + kh) * dh, voff = (size_t)(nh + nkv + kh) * dh;
  float m = -INFINITY, l = 0.f;
  float o[kDhSlots];
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) o[t] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float sc = -INFINITY;
    if (j <= i) {
      const size_t rk = (row0 + j) * ld + koff;
      float a = 0.f;
      for (int c = 0; c < dh; ++c) a = fmaf(qs[c], ldf(qkv, rk + c), a);
      sc = a;
    }
    const float nm = fmaxf(m, wave_max(sc));
    const float corr = __expf(m - nm);  // first chunk: exp(-inf) = 0
    const float pj = (j <= i) ? __expf(sc - nm) : 0.f;
    l = l * corr + wave_sum(pj);
    m = nm;
    __syncthreads();
    ps[lane] = pj;
    __syncthreads();
    const int jn = min(64, i - j0 + 1);
#pragma unroll
    for (int t = 0; t < kDhSlots; ++t) {
      const int c = lane + 64 * t;
      if (c < dh) {
        float a = o[t] * corr;
        for (int jj = 0; jj < jn; ++jj)
          a = fmaf(ps[jj], ldf(qkv, (row0 + j0 + jj) * ld + voff + c), a);
        o[t] = a;
      }
    }
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) {
    const int c = lane + 64 * t;
    if (c < dh) stf(out, (row0 + i) * ((size_t)nh * dh) + (size_t)h * dh + c, o[t] * inv);
  }
  if (lane == 0) lse[stat_index(cu, Trows, sv, b, h, nh, Smax, i)] = m + logf(l);
}

// delta[b,h,i] = sum_c dO[i,h,c] * O[i,h,c]
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_kernel(const T* __restrict__ out, const T* __restrict__ dout,
                                                        float* __restrict__ delta, int Smax, int nh, int dh,
                                                        const int* __restrict__ cu, int64_t Trows) {
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const SeqView sv = seq_view(cu, b, Smax, Trows);
  if (i >= sv.len) return;
  const size_t row0 = (size_t)sv.row0;
  const size_t base = (row0 + i) * ((size_t)nh * dh) + (size_t)h * dh;
  float a = 0.f;
  for (int c = threadIdx.x; c < dh; c += 64) a += ldf(out, base + c) * ldf(dout, base + c);
  a = wave_sum(a);
  if (threadIdx.x == 0) delta[stat_index(cu, Trows, sv, b, h, nh, Smax, i)] = a;
}

// The same for head sizes whose 16-byte pieces form a power-of-two group of lanes (8 <= dh <= 512): one
// block per row, 8 channels per lane, the dh/8 lanes of a head combine by shuffles.
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_vec_kernel(const T* __restrict__ out, const T* __restrict__ dout,
                                                             float* __restrict__ delta, int Smax, int nh, int dh,
                                                             const int* __restrict__ cu, int64_t Trows) {
  const int i = blockIdx.x, b = blockIdx.y;
  const SeqView sv = seq_view(cu, b, Smax, Trows);
  if (i >= sv.len) return;
  const int lph = dh >> 3;                         // lanes per head
  const int width = nh * dh;
  const size_t base = ((size_t)sv.row0 + i) * (size_t)width;
  for (int c0 = 0; c0 < width; c0 += 256 * 8) {    // uniform trip count: the shuffles below are wave-wide
    const int c = c0 + (int)threadIdx.x * 8;
    float a = 0.f;
    if (c < width) {
      float o[8], g[8];
      ld8(out, base + c, o);
      ld8(dout, base + c, g);
#pragma unroll
      for (int j = 0; j < 8; ++j) a += o[j] * g[j];
    }
    for (int off = lph >> 1; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
    if (c < width && (threadIdx.x & (lph - 1)) == 0) delta[stat_index(cu, Trows, sv, b, c / dh, nh, Smax, i)] = a;
  }
}

template <typename T>
__global__ __launch_bounds__(64) void attn_dq_simple_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ delta, T* __restrict__ dqkv,
                                                            int Smax, int nh, int nkv, int dh,
                                                            const int* __restrict__ cu, int64_t Trows) {
  __shared__ float qs[kMaxDh], dos[kMaxDh];
  __shared__ float dss[64];
  const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const SeqView sv = seq_view(cu, b, Smax, Trows);
  if (i >= sv.len) return;
  const size_t row0 = (size_t)sv.row0;
  const int lane = threadIdx.x;
  const int G = nh / nkv, kh = h / G;
  const int ld = (nh + 2 * nkv) * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t rowq = (row0 + i) * ld;
  const size_t rowo = (row0 + i) * ((size_t)nh * dh) + (size_t)h * dh;
  for (int c = lane; c < dh; c += 64) {
    qs[c] = ldf(qkv, rowq + (size_t)h * dh + c) * scale;
    dos[c] = ldf(dout, rowo + c);
  }
  __syncthreads();
  const size_t koff = (size_t)(nh + kh) * dh, voff = (size_t)(nh + nkv + kh) * dh;
  const float L = lse[stat_index(cu, Trows, sv, b, h, nh, Smax, i)];
  const float D = delta[stat_index(cu, Trows, sv, b, h, nh, Smax, i)];
  float dq[kDhSlots];
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) dq[t] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float ds = 0.f;
    if (j <= i) {
      const size_t rk = (row0 + j) * ld;
      float a = 0.f, dp = 0.f;
      for (int c = 0; c < dh; ++c) {
        a = fmaf(qs[c], ldf(qkv, rk + koff + c), a);
        dp = fmaf(dos[c], ldf(qkv, rk + voff + c), dp);
      }
      ds = __expf(a - L) * (dp - D);
    }
    __syncthreads();
    dss[lane] = ds;
    __syncthreads();
    const int jn = min(64, i - j0 + 1);
#pragma unroll
    for (int t = 0; t < kDhSlots; ++t) {
      const int c = lane + 64 * t;
      if (c < dh) {
        float a = dq[t];
        for (int jj = 0; jj < jn; ++jj)
          a = fmaf(dss[jj], ldf(qkv, (row0 + j0 + jj) * ld + koff + c), a);
        dq[t] = a;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) {
    const int c = lane + 64 * t;
    if (c < dh) stf(dqkv, rowq + (size_t)h * dh + c, dq[t] * scale);
  }
}

template <typename T>
__global__ __launch_bounds__(64) void attn_dkv_simple_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ delta, T* __restrict__ dqkv,
                                                             int Smax, int nh, int nkv, int dh,
                                                             const int* __restrict__ cu, int64_t Trows) {
  __shared__ float ks[kMaxDh], vs[kMaxDh];
  __shared__ float pss[64], dss[64];
  const int j = blockIdx.x, kh = blockIdx.y, b = blockIdx.z;
  const SeqView sv = seq_view(cu, b, Smax, Trows);
  const int S = sv.len;
  if (j >= S) return;
  const size_t row0 = (size_t)sv.row0;
  const int lane = threadIdx.x;
  const int G = nh / nkv;
  const int ld = (nh + 2 * nkv) * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t koff = (size_t)(nh + kh) * dh, voff = (size_t)(nh + nkv + kh) * dh;
  const size_t rowk = (row0 + j) * ld;
  for (int c = lane; c < dh; c += 64) {
    ks[c] = ldf(qkv, rowk + koff + c) * scale;
    vs[c] = ldf(qkv, rowk + voff + c);
  }
  __syncthreads();
  float dk[kDhSlots], dv[kDhSlots];
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) dk[t] = dv[t] = 0.f;
  for (int g = 0; g < G; ++g) {
    const int h = kh * G + g;
    for (int i0 = j; i0 < S; i0 += 64) {
      const int i = i0 + lane;
      float pv = 0.f, ds = 0.f;
      if (i < S) {
        const size_t rq = (row0 + i) * ld + (size_t)h * dh;
        const size_t ro = (row0 + i) * ((size_t)nh * dh) + (size_t)h * dh;
        float a = 0.f, dp = 0.f;
        for (int c = 0; c < dh; ++c) {
          a = fmaf(ks[c], ldf(qkv, rq + c), a);
          dp = fmaf(vs[c], ldf(dout, ro + c), dp);
        }
        pv = __expf(a - lse[stat_index(cu, Trows, sv, b, h, nh, Smax, i)]);
        ds = pv * (dp - delta[stat_index(cu, Trows, sv, b, h, nh, Smax, i)]);
      }
      __syncthreads();
      pss[lane] = pv;
      dss[lane] = ds;
      __syncthreads();
      const int in = min(64, S - i0);
#pragma unroll
      for (int t = 0; t < kDhSlots; ++t) {
        const int c = lane + 64 * t;
        if (c < dh) {
          float a = dv[t], bb = dk[t];
          for (int ii = 0; ii < in; ++ii) {
            const size_t rq = (row0 + i0 + ii) * ld + (size_t)h * dh;
            const size_t ro = (row0 + i0 + ii) * ((size_t)nh * dh) + (size_t)h * dh;
            a = fmaf(pss[ii], ldf(dout, ro + c), a);
            bb = fmaf(dss[ii], ldf(qkv, rq + c), bb);
          }
          dv[t] = a;
          dk[t] = bb;
        }
      }
    }
  }
#pragma unroll
  for (int t = 0; t < kDhSlots; ++t) {
    const int c = lane + 64 * t;
    if (c < dh) {
      stf(dqkv, rowk + koff + c, dk[t] * scale);
      stf(dqkv, rowk + voff + c, dv[t]);
    }
  }
}

static bool simple_ok(const AttnArgs& a) {
  return a.dh <= kMaxDh && a.B <= 65535 && a.nh <= 65535 && a.S > 0 && a.B > 0;
}

hipError_t launch_attn_fwd_simple(const AttnArgs& a, hipStream_t s) {
  if (!simple_ok(a)) return hipErrorInvalidValue;
  ProfScope ps("attn_fwd_simple", 2.0 * a.B * a.nh * a.dh * (double)a.S * (a.S + 1), 0, s);
  dim3 grid(a.S, a.nh, a.B), blk(64);
  if (a.dtype == kBF16) hipLaunchKernelGGL(attn_fwd_simple_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)a.qkv, (bf16_t*)a.out, a.lse, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
  else hipLaunchKernelGGL(attn_fwd_simple_kernel<float>, grid, blk, 0, s, (const float*)a.qkv, (float*)a.out, a.lse, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
  return hipGetLastError();
}

hipError_t launch_attn_delta(const AttnArgs& a, hipStream_t s) {
  ProfScope ps("attn_delta", 0, 2.0 * a.B * a.S * a.nh * a.dh * dtype_size(a.dtype), s);
  const int lph = a.dh / 8;
  if (a.dh % 8 == 0 && lph >= 1 && lph <= 64 && (lph & (lph - 1)) == 0 &&
      (((uintptr_t)a.out | (uintptr_t)a.dout) & 15) == 0) {
    dim3 grid(a.S, a.B), blk(256);
    if (a.dtype == kBF16) hipLaunchKernelGGL(attn_delta_vec_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)a.out, (const bf16_t*)a.dout, a.delta, a.S, a.nh, a.dh, a.cu_seqlens, a.total_rows);
    else hipLaunchKernelGGL(attn_delta_vec_kernel<float>, grid, blk, 0, s, (const float*)a.out, (const float*)a.dout, a.delta, a.S, a.nh, a.dh, a.cu_seqlens, a.total_rows);
    return hipGetLastError();
  }
  dim3 grid(a.S, a.nh, a.B), blk(64);
  if (a.dtype == kBF16) hipLaunchKernelGGL(attn_delta_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)a.out, (const bf16_t*)a.dout, a.delta, a.S, a.nh, a.dh, a.cu_seqlens, a.total_rows);
  else hipLaunchKernelGGL(attn_delta_kernel<float>, grid, blk, 0, s, (const float*)a.out, (const float*)a.dout, a.delta, a.S, a.nh, a.dh, a.cu_seqlens, a.total_rows);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(const AttnArgs& a, hipStream_t s) {
  if (!simple_ok(a)) return hipErrorInvalidValue;
  hipError_t e = launch_attn_delta(a, s);
  if (e != hipSuccess) return e;
  ProfScope ps("attn_bwd_simple", 7.0 * a.B * a.nh * a.dh * (double)a.S * (a.S + 1), 0, s);
  dim3 gq(a.S, a.nh, a.B), gk(a.S, a.nkv, a.B), blk(64);
  if (a.dtype == kBF16) {
    hipLaunchKernelGGL(attn_dq_simple_kernel<bf16_t>, gq, blk, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse, a.delta, (bf16_t*)a.dqkv, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
    hipLaunchKernelGGL(attn_dkv_simple_kernel<bf16_t>, gk, blk, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dout, a.lse, a.delta, (bf16_t*)a.dqkv, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
  } else {
    hipLaunchKernelGGL(attn_dq_simple_kernel<float>, gq, blk, 0, s, (const float*)a.qkv, (const float*)a.dout, a.lse, a.delta, (float*)a.dqkv, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
    hipLaunchKernelGGL(attn_dkv_simple_kernel<float>, gk, blk, 0, s, (const float*)a.qkv, (const float*)a.dout, a.lse, a.delta, (float*)a.dqkv, a.S, a.nh, a.nkv, a.dh, a.cu_seqlens, a.total_rows);
  }
  return hipGetLastError();
}

}  // namespace tide

// Kernels of the multi-step unroll of the draft (Sec. 3.2 names EAGLE-3 as the draft architecture, Sec. 5.1
// fixes gamma = 3 draft tokens per round): from its second draft token on the draft is fed its own layer
// output in place of a captured feature.  Row i of step s stands for position i + s - 1; it attends to the
// step-1 keys/values of rows 0..i (the ordinary causal attention, run by the flash kernels on a buffer that
// holds the step's queries next to the step-1 keys and values) and to the ONE key/value it produced itself
// at each of the steps 2..s.  Those few extra pairs per row are merged into the flash result here, one
// wavefront per (row, query head): HBM-bound streaming work, no contraction.
#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

// tokens / mask / input ids of step `shift + 1`: moved left by `shift` inside every sequence (label -1, mask 0,
// id -1 where the position leaves the sequence), and sel = 1 for every row that carries loss at this or a
// later step (its layer output is needed: for its own logits or as the next step's feature).
__global__ __launch_bounds__(256) void shift_inputs_kernel(const int32_t* __restrict__ tokens,
                                                           const uint8_t* __restrict__ mask,
                                                           const int32_t* __restrict__ ids, int64_t T, int S, int V,
                                                           int shift, int n_steps, int32_t* __restrict__ tokens_s,
                                                           uint8_t* __restrict__ mask_s, uint8_t* __restrict__ sel_s,
                                                           int32_t* __restrict__ ids_s, const int* __restrict__ cu,
                                                           int nseq) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  // end = one past the last row of the sequence that owns row t (t itself for a padding row of a packed batch)
  int64_t end;
  if (cu) {
    const int64_t c0 = min(max((int64_t)cu[0], (int64_t)0), T), cN = min(max((int64_t)cu[nseq], c0), T);
    if (t < c0 || t >= cN) {
      end = t;
    } else {
      int lo = 0, hi = nseq;               // largest b with cu[b] <= t
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
      }
      end = min(max((int64_t)cu[lo + 1], t + 1), cN);   // inside the buffers whatever the offsets hold
    }
  } else {
    end = (t / S + 1) * (int64_t)S;
  }
  const bool in = t + shift < end;
  tokens_s[t] = in ? tokens[t + shift] : -1;
  mask_s[t] = in ? mask[t + shift] : (uint8_t)0;
  if (ids_s) ids_s[t] = in ? ids[t + shift] : -1;
  int sel = 0;
  for (int j = shift; j < n_steps && t + j < end; ++j) {
    const int tk = tokens[t + j];
    if (mask[t + j] != 0 && tk >= 0 && tk < V) sel = 1;
  }
  sel_s[t] = (uint8_t)sel;
}

hipError_t launch_shift_inputs(const int32_t* tokens, const uint8_t* mask, const int32_t* ids, int64_t T, int S, int V,
                               int shift, int n_steps, int32_t* tokens_s, uint8_t* mask_s, uint8_t* sel_s,
                               int32_t* ids_s, const int* cu, int nseq, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipLaunchKernelGGL(shift_inputs_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, tokens, mask, ids, T, S, V, shift, n_steps, tokens_s, mask_s, sel_s, ids_s, cu, nseq);
  return hipGetLastError();
}

// own[t] = key and value columns of qkv[t] (this step's own pair, after RoPE), which are then overwritten
// by those of qkv1[t] (step 1), so that the flash kernels find the step's queries beside the step-1 keys/values
template <typename T>
__global__ __launch_bounds__(256) void kv_swap_kernel(T* __restrict__ qkv, const T* __restrict__ qkv1,
                                                      T* __restrict__ own, int nq, int nkv2, int ld) {
  const size_t t = blockIdx.x;
  T* row = qkv + t * (size_t)ld + nq;
  const T* row1 = qkv1 + t * (size_t)ld + nq;
  T* o = own + t * (size_t)nkv2;
  for (int e = threadIdx.x; e < nkv2; e += 256) {
    o[e] = row[e];
    row[e] = row1[e];
  }
}

hipError_t launch_kv_swap(int64_t T, int nq, int nk, void* qkv, const void* qkv1, void* own, int dtype, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps("kv_swap", 0, 6.0 * (double)T * nk * dtype_size(dtype), s);
  const int ld = nq + 2 * nk;
  if (dtype == kBF16) hipLaunchKernelGGL(kv_swap_kernel<bf16_t>, dim3((unsigned)T), dim3(256), 0, s, (bf16_t*)qkv, (const bf16_t*)qkv1, (bf16_t*)own, nq, 2 * nk, ld);
  else hipLaunchKernelGGL(kv_swap_kernel<float>, dim3((unsigned)T), dim3(256), 0, s, (float*)qkv, (const float*)qkv1, (float*)own, nq, 2 * nk, ld);
  return hipGetLastError();
}

namespace {
constexpr int kMaxDhPerLane = 4;   // head_dim <= 256
}  // namespace

// out[t, h] and lse[b, h, i] hold the causal attention of the step's query over the step-1 keys/values.  With
// s_j = scale * q . k_j for the n_own own pairs:  L = log(exp(lse) + sum_j exp(s_j)),
// out <- exp(lse - L) out + sum_j exp(s_j - L) v_j,  lse <- L   (one softmax over prefix and own pairs).
template <typename T>
__global__ __launch_bounds__(256) void own_kv_merge_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ out,
                                                               float* __restrict__ lse, OwnKV own, int n_own,
                                                               int64_t n_pairs, int nh, int nkv, int dh, int S,
                                                               float scale, int64_t packed_T) {
  const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= n_pairs) return;   // whole wavefronts leave; no barrier below
  const int lane = threadIdx.x & 63;
  const int64_t t = wid / nh;
  const int h = (int)(wid % nh), kh = h / (nh / nkv);
  const int nq = nh * dh, nk = nkv * dh;
  const T* q = qkv + (size_t)t * (nq + 2 * nk) + (size_t)h * dh;
  float qv[kMaxDhPerLane];
#pragma unroll
  for (int c = 0; c < kMaxDhPerLane; ++c) {
    const int e = lane + 64 * c;
    qv[c] = e < dh ? ldf(q, e) : 0.f;
  }
  float sc[kMaxUnroll];
  for (int j = 0; j < n_own; ++j) {
    const T* kj = (const T*)own.kv[j] + (size_t)t * (2 * nk) + (size_t)kh * dh;
    float part = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxDhPerLane; ++c) {
      const int e = lane + 64 * c;
      if (e < dh) part += qv[c] * ldf(kj, e);
    }
    sc[j] = scale * wave_sum(part);
  }
  // lse is [B, nh, S] in the fixed layout and [nh, T] for a packed batch
  const size_t li = packed_T ? (size_t)h * (size_t)packed_T + (size_t)t : ((size_t)(t / S) * nh + h) * (size_t)S + (size_t)(t % S);
  const float l0 = lse[li];
  float m = l0;
  for (int j = 0; j < n_own; ++j) m = fmaxf(m, sc[j]);
  float sum = expf(l0 - m);
  for (int j = 0; j < n_own; ++j) sum += expf(sc[j] - m);
  const float L = m + logf(sum);
  const float w0 = expf(l0 - L);
  T* o = out + (size_t)t * nq + (size_t)h * dh;
#pragma unroll
  for (int c = 0; c < kMaxDhPerLane; ++c) {
    const int e = lane + 64 * c;
    if (e < dh) {
      float acc = w0 * ldf(o, e);
      for (int j = 0; j < n_own; ++j) {
        const T* vj = (const T*)own.kv[j] + (size_t)t * (2 * nk) + nk + (size_t)kh * dh;
        acc += expf(sc[j] - L) * ldf(vj, e);
      }
      stf(o, e, acc);
    }
  }
  if (lane == 0) lse[li] = L;
}

// Same merge with 8 consecutive elements per lane (16-byte accesses in bf16): LPH = head_dim / 8 lanes serve one
// (row, query head), 64 / LPH heads share a wavefront; reductions run inside the LPH-lane group.
template <typename T, int LPH>
__global__ __launch_bounds__(256) void own_kv_merge_fwd_vec_kernel(const T* __restrict__ qkv, T* __restrict__ out,
                                                                   float* __restrict__ lse, OwnKV own, int n_own,
                                                                   int64_t n_pairs, int nh, int nkv, int S, float scale,
                                                                   int64_t packed_T) {
  constexpr int HPW = 64 / LPH, dh = LPH * 8;
  const int lane = threadIdx.x & 63, sub = lane % LPH;
  const int64_t pair = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * HPW + lane / LPH;
  const bool live = pair < n_pairs;
  const int64_t t = live ? pair / nh : 0;
  const int h = live ? (int)(pair % nh) : 0, kh = h / (nh / nkv);
  const int nq = nh * dh, nk = nkv * dh;
  const size_t qo = (size_t)t * (nq + 2 * nk) + (size_t)h * dh + sub * 8;
  const size_t ko = (size_t)t * (2 * nk) + (size_t)kh * dh + sub * 8;
  float qv[8];
  ld8(qkv, qo, qv);
  float sc[kMaxUnroll];
  for (int j = 0; j < n_own; ++j) {
    float kv[8];
    ld8((const T*)own.kv[j], ko, kv);
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) part += qv[e] * kv[e];
#pragma unroll
    for (int o = LPH / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
    sc[j] = scale * part;
  }
  const size_t li = packed_T ? (size_t)h * (size_t)packed_T + (size_t)t : ((size_t)(t / S) * nh + h) * (size_t)S + (size_t)(t % S);
  const float l0 = lse[li];
  float m = l0;
  for (int j = 0; j < n_own; ++j) m = fmaxf(m, sc[j]);
  float sum = expf(l0 - m);
  for (int j = 0; j < n_own; ++j) sum += expf(sc[j] - m);
  const float L = m + logf(sum);
  const float w0 = expf(l0 - L);
  const size_t oo = (size_t)t * nq + (size_t)h * dh + sub * 8;
  float acc[8];
  ld8(out, oo, acc);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] *= w0;
  for (int j = 0; j < n_own; ++j) {
    float vv[8];
    ld8((const T*)own.kv[j], ko + nk, vv);
    const float wj = expf(sc[j] - L);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += wj * vv[e];
  }
  if (live) {
    st8(out, oo, acc);
    if (sub == 0) lse[li] = L;
  }
}

hipError_t launch_own_kv_merge_fwd(int64_t T, int S, int nh, int nkv, int dh, const void* qkv, void* out, float* lse,
                                   const OwnKV& own, int n_own, int packed, int dtype, hipStream_t s) {
  const int64_t n_pairs = T * nh;
  const int64_t packed_T = packed ? T : 0;
  if (n_pairs <= 0 || n_own <= 0) return hipSuccess;
  if (n_own > kMaxUnroll || dh > 64 * kMaxDhPerLane || nh % nkv) return hipErrorInvalidValue;
  ProfScope ps("own_kv_merge_fwd", 0, (double)n_pairs * dh * (3.0 + 2.0 * n_own) * dtype_size(dtype), s);
  const float scale = 1.0f / sqrtf((float)dh);
  const bool aligned = (((uintptr_t)qkv | (uintptr_t)out) & 15) == 0;
  bool own_aligned = true;
  for (int j = 0; j < n_own; ++j) own_aligned = own_aligned && (((uintptr_t)own.kv[j]) & 15) == 0;
  if ((dh == 128 || dh == 64) && aligned && own_aligned) {
    const int hpw = dh == 128 ? 4 : 8;   // (row, head) pairs per wavefront
    dim3 gridv((unsigned)((n_pairs + 4 * hpw - 1) / (4 * hpw))), blkv(256);
#define TIDE_MERGE_FWD(T, LPH) hipLaunchKernelGGL((own_kv_merge_fwd_vec_kernel<T, LPH>), gridv, blkv, 0, s, (const T*)qkv, (T*)out, lse, own, n_own, n_pairs, nh, nkv, S, scale, packed_T)
    if (dtype == kBF16) { if (dh == 128) TIDE_MERGE_FWD(bf16_t, 16); else TIDE_MERGE_FWD(bf16_t, 8); }
    else { if (dh == 128) TIDE_MERGE_FWD(float, 16); else TIDE_MERGE_FWD(float, 8); }
#undef TIDE_MERGE_FWD
    return hipGetLastError();
  }
  dim3 grid((unsigned)((n_pairs + 3) / 4)), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(own_kv_merge_fwd_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)qkv, (bf16_t*)out, lse, own, n_own, n_pairs, nh, nkv, dh, S, scale, packed_T);
  else hipLaunchKernelGGL(own_kv_merge_fwd_kernel<float>, grid, blk, 0, s, (const float*)qkv, (float*)out, lse, own, n_own, n_pairs, nh, nkv, dh, S, scale, packed_T);
  return hipGetLastError();
}

// Backward of the merge, one wavefront per (row, key/value head), which owns the group of query heads that read
// the pair.  With L, delta = rowsum(dO * O) of the merged result, for own pair j and query head h:
//   p = exp(s_j - L),  ds = p * (dO_h . v_j - delta_h),
//   dq_h += scale ds k_j,  dk_j += scale ds q_h,  dv_j += p dO_h.
// dq is added to what the flash backward wrote into dqkv; (dk_j, dv_j) go to the pair's own gradient buffer,
// written if first (the last step of the unroll, which reads every pair, runs its backward first), else added.
template <typename T>
__global__ __launch_bounds__(256) void own_kv_merge_bwd_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta, OwnKV own,
                                                               OwnKVGrad grad, int n_own, int first, T* __restrict__ dqkv,
                                                               int64_t n_pairs, int nh, int nkv, int dh, int S,
                                                               float scale, int64_t packed_T) {
  const int64_t wid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wid >= n_pairs) return;   // whole wavefronts leave; no barrier below
  const int lane = threadIdx.x & 63;
  const int64_t t = wid / nkv;
  const int kh = (int)(wid % nkv), G = nh / nkv;
  const int nq = nh * dh, nk = nkv * dh, ld = nq + 2 * nk;
  // lse / delta: [B, nh, S] in the fixed layout, [nh, T] for a packed batch; index = stat0 + h * stat_h
  const size_t stat0 = packed_T ? (size_t)t : ((size_t)(t / S) * nh) * (size_t)S + (size_t)(t % S);
  const size_t stat_h = packed_T ? (size_t)packed_T : (size_t)S;
  for (int j = 0; j < n_own; ++j) {
    const T* kj = (const T*)own.kv[j] + (size_t)t * (2 * nk) + (size_t)kh * dh;
    const T* vj = kj + nk;
    float kv[kMaxDhPerLane], vv[kMaxDhPerLane], dk[kMaxDhPerLane], dv[kMaxDhPerLane];
#pragma unroll
    for (int c = 0; c < kMaxDhPerLane; ++c) {
      const int e = lane + 64 * c;
      kv[c] = e < dh ? ldf(kj, e) : 0.f;
      vv[c] = e < dh ? ldf(vj, e) : 0.f;
      dk[c] = dv[c] = 0.f;
    }
    for (int g = 0; g < G; ++g) {
      const int h = kh * G + g;
      const T* q = qkv + (size_t)t * ld + (size_t)h * dh;
      const T* dO = dout + (size_t)t * nq + (size_t)h * dh;
      T* dq = dqkv + (size_t)t * ld + (size_t)h * dh;
      float qv[kMaxDhPerLane], dov[kMaxDhPerLane];
      float sp = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < kMaxDhPerLane; ++c) {
        const int e = lane + 64 * c;
        qv[c] = e < dh ? ldf(q, e) : 0.f;
        dov[c] = e < dh ? ldf(dO, e) : 0.f;
        sp += qv[c] * kv[c];
        dp += dov[c] * vv[c];
      }
      sp = scale * wave_sum(sp);
      dp = wave_sum(dp);
      const size_t li = stat0 + (size_t)h * stat_h;
      const float p = expf(sp - lse[li]);
      const float ds = p * (dp - delta[li]);
#pragma unroll
      for (int c = 0; c < kMaxDhPerLane; ++c) {
        const int e = lane + 64 * c;
        if (e < dh) stf(dq, e, ldf(dq, e) + scale * ds * kv[c]);
        dk[c] += scale * ds * qv[c];
        dv[c] += p * dov[c];
      }
    }
    T* gk = (T*)grad.kv[j] + (size_t)t * (2 * nk) + (size_t)kh * dh;
    T* gv = gk + nk;
#pragma unroll
    for (int c = 0; c < kMaxDhPerLane; ++c) {
      const int e = lane + 64 * c;
      if (e < dh) {
        stf(gk, e, first ? dk[c] : ldf(gk, e) + dk[c]);
        stf(gv, e, first ? dv[c] : ldf(gv, e) + dv[c]);
      }
    }
  }
}

// The same backward with 8 consecutive elements per lane: LPH = head_dim / 8 lanes serve one (row, key/value head).
template <typename T, int LPH>
__global__ __launch_bounds__(256) void own_kv_merge_bwd_vec_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                                   const float* __restrict__ lse,
                                                                   const float* __restrict__ delta, OwnKV own,
                                                                   OwnKVGrad grad, int n_own, int first,
                                                                   T* __restrict__ dqkv, int64_t n_pairs, int nh, int nkv,
                                                                   int S, float scale, int64_t packed_T) {
  constexpr int PPW = 64 / LPH, dh = LPH * 8;
  const int lane = threadIdx.x & 63, sub = lane % LPH;
  const int64_t pair = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * PPW + lane / LPH;
  const bool live = pair < n_pairs;
  const int64_t t = live ? pair / nkv : 0;
  const int kh = live ? (int)(pair % nkv) : 0, G = nh / nkv;
  const int nq = nh * dh, nk = nkv * dh, ld = nq + 2 * nk;
  const size_t stat0 = packed_T ? (size_t)t : ((size_t)(t / S) * nh) * (size_t)S + (size_t)(t % S);
  const size_t stat_h = packed_T ? (size_t)packed_T : (size_t)S;
  const size_t ko = (size_t)t * (2 * nk) + (size_t)kh * dh + sub * 8;
  for (int j = 0; j < n_own; ++j) {
    float kv[8], vv[8], dk[8], dv[8];
    ld8((const T*)own.kv[j], ko, kv);
    ld8((const T*)own.kv[j], ko + nk, vv);
#pragma unroll
    for (int e = 0; e < 8; ++e) dk[e] = dv[e] = 0.f;
    for (int g = 0; g < G; ++g) {
      const int h = kh * G + g;
      const size_t qo = (size_t)t * ld + (size_t)h * dh + sub * 8;
      float qv[8], dov[8], dq[8];
      ld8(qkv, qo, qv);
      ld8(dout, (size_t)t * nq + (size_t)h * dh + sub * 8, dov);
      float sp = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { sp += qv[e] * kv[e]; dp += dov[e] * vv[e]; }
#pragma unroll
      for (int o = LPH / 2; o > 0; o >>= 1) { sp += __shfl_xor(sp, o, 64); dp += __shfl_xor(dp, o, 64); }
      const size_t li = stat0 + (size_t)h * stat_h;
      const float p = expf(scale * sp - lse[li]);
      const float ds = p * (dp - delta[li]);
      ld8(dqkv, qo, dq);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        dq[e] += scale * ds * kv[e];
        dk[e] += scale * ds * qv[e];
        dv[e] += p * dov[e];
      }
      if (live) st8(dqkv, qo, dq);
    }
    T* gbuf = (T*)grad.kv[j];
    if (!first) {
      float ok[8], ov[8];
      ld8(gbuf, ko, ok);
      ld8(gbuf, ko + nk, ov);
#pragma unroll
      for (int e = 0; e < 8; ++e) { dk[e] += ok[e]; dv[e] += ov[e]; }
    }
    if (live) {
      st8(gbuf, ko, dk);
      st8(gbuf, ko + nk, dv);
    }
  }
}

hipError_t launch_own_kv_merge_bwd(int64_t T, int S, int nh, int nkv, int dh, const void* qkv, const void* dout,
                                   const float* lse, const float* delta, const OwnKV& own, const OwnKVGrad& grad,
                                   int n_own, int first, void* dqkv, int packed, int dtype, hipStream_t s) {
  const int64_t n_pairs = T * nkv;
  const int64_t packed_T = packed ? T : 0;
  if (n_pairs <= 0 || n_own <= 0) return hipSuccess;
  if (n_own > kMaxUnroll || dh > 64 * kMaxDhPerLane || nh % nkv) return hipErrorInvalidValue;
  ProfScope ps("own_kv_merge_bwd", 0, (double)T * nh * dh * (4.0 * n_own) * dtype_size(dtype), s);
  const float scale = 1.0f / sqrtf((float)dh);
  bool aligned = (((uintptr_t)qkv | (uintptr_t)dout | (uintptr_t)dqkv) & 15) == 0;
  for (int j = 0; j < n_own; ++j) aligned = aligned && ((((uintptr_t)own.kv[j]) | ((uintptr_t)grad.kv[j])) & 15) == 0;
  if ((dh == 128 || dh == 64) && aligned) {
    const int ppw = dh == 128 ? 4 : 8;   // (row, key/value head) pairs per wavefront
    dim3 gridv((unsigned)((n_pairs + 4 * ppw - 1) / (4 * ppw))), blkv(256);
#define TIDE_MERGE_BWD(T, LPH) hipLaunchKernelGGL((own_kv_merge_bwd_vec_kernel<T, LPH>), gridv, blkv, 0, s, (const T*)qkv, (const T*)dout, lse, delta, own, grad, n_own, first, (T*)dqkv, n_pairs, nh, nkv, S, scale, packed_T)
    if (dtype == kBF16) { if (dh == 128) TIDE_MERGE_BWD(bf16_t, 16); else TIDE_MERGE_BWD(bf16_t, 8); }
    else { if (dh == 128) TIDE_MERGE_BWD(float, 16); else TIDE_MERGE_BWD(float, 8); }
#undef TIDE_MERGE_BWD
    return hipGetLastError();
  }
  dim3 grid((unsigned)((n_pairs + 3) / 4)), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(own_kv_merge_bwd_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)qkv, (const bf16_t*)dout, lse, delta, own, grad, n_own, first, (bf16_t*)dqkv, n_pairs, nh, nkv, dh, S, scale, packed_T);
  else hipLaunchKernelGGL(own_kv_merge_bwd_kernel<float>, grid, blk, 0, s, (const float*)qkv, (const float*)dout, lse, delta, own, grad, n_own, first, (float*)dqkv, n_pairs, nh, nkv, dh, S, scale, packed_T);
  return hipGetLastError();
}

// Key/value columns of a step's dqkv after the flash backward: for a later step they hold its share of the
// STEP-1 key/value gradient.  mode 0: acc1 = them (first share), mode 1: acc1 += them; both then put the step's
// own pair gradient (own_grad) in their place.  mode 2 (step 1 itself): them += acc1.
template <typename T>
__global__ __launch_bounds__(256) void kv_grad_route_kernel(T* __restrict__ dqkv, T* __restrict__ acc1,
                                                            const T* __restrict__ own_grad, int nq, int nkv2, int ld,
                                                            int mode) {
  const size_t t = blockIdx.x;
  T* row = dqkv + t * (size_t)ld + nq;
  T* a = acc1 + t * (size_t)nkv2;
  for (int e = threadIdx.x; e < nkv2; e += 256) {
    const float v = ldf(row, e);
    if (mode == 2) {
      stf(row, e, v + ldf(a, e));
    } else {
      stf(a, e, mode == 0 ? v : v + ldf(a, e));
      row[e] = own_grad[t * (size_t)nkv2 + e];
    }
  }
}

hipError_t launch_kv_grad_route(int64_t T, int nq, int nk, void* dqkv, void* acc1, const void* own_grad, int mode,
                                int dtype, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  if (mode < 0 || mode > 2 || (mode != 2 && !own_grad)) return hipErrorInvalidValue;
  ProfScope ps("kv_grad_route", 0, 8.0 * (double)T * nk * dtype_size(dtype), s);
  const int ld = nq + 2 * nk;
  if (dtype == kBF16) hipLaunchKernelGGL(kv_grad_route_kernel<bf16_t>, dim3((unsigned)T), dim3(256), 0, s, (bf16_t*)dqkv, (bf16_t*)acc1, (const bf16_t*)own_grad, nq, 2 * nk, ld, mode);
  else hipLaunchKernelGGL(kv_grad_route_kernel<float>, dim3((unsigned)T), dim3(256), 0, s, (float*)dqkv, (float*)acc1, (const float*)own_grad, nq, 2 * nk, ld, mode);
  return hipGetLastError();
}

}  // namespace tide

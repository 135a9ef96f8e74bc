// HBM-bound kernels of the TIDE draft-training step for gfx950: mask count, RMSNorm forward and
// backward, RoPE, SwiGLU, cross-entropy row statistics and logit gradient, loss reduction, fused AdamW.
// All are coalesced 16-byte-per-lane streaming kernels with 64-wide wavefront reductions; arithmetic is
// fp32 whatever the storage type.
#include "kernels.h"
#include "prof.h"
#include "tide_common.h"

namespace tide {

// ----------------------------------------------------------------------------------------------
// Row plan: N = max(1, #keep) with keep_t = mask_t != 0 and 0 <= token_t < V, the ascending list of the
// selected rows (the kept rows; every row when select_all is set, which the forward pass with arg-max
// output needs) and its inverse row_pos (-1 for rows not selected).  A row that carries no loss reaches
// the loss and the gradients only through its key and value, so everything after the attention runs on
// the selected rows alone.  Integer counts and a fixed order: deterministic.
// ----------------------------------------------------------------------------------------------
// Two launches of 1024-thread blocks, one row per thread: block-wise counts, then every block finds its
// offset from the counts of the blocks before it and writes its rows (a single block walking all rows took
// 0.11 ms at 32768 rows, at the head of every call).
namespace {
struct RowFlags { int keep, sel; };
__device__ __forceinline__ RowFlags row_flags(const int32_t* tokens, const uint8_t* mask, int64_t t, int64_t T, int V,
                                              int select_all, int64_t v0, int64_t v1, const uint8_t* sel_mask) {
  RowFlags f{0, 0};
  if (t < T) {
    const int tk = tokens[t];
    f.keep = (mask[t] != 0 && tk >= 0 && tk < V && t >= v0 && t < v1) ? 1 : 0;
    f.sel = sel_mask ? (sel_mask[t] != 0 ? 1 : 0) : (select_all ? 1 : f.keep);
  }
  return f;
}
}  // namespace

__global__ __launch_bounds__(1024) void plan_count_kernel(const int32_t* __restrict__ tokens,
                                                          const uint8_t* __restrict__ mask, int64_t T, int V,
                                                          int select_all, const int* __restrict__ cu, int nseq,
                                                          int* __restrict__ blk_counts,
                                                          const uint8_t* __restrict__ sel_mask) {
  __shared__ int ws_sel[16], ws_keep[16];
  // packed batches: only rows inside [cu[0], cu[nseq]) belong to a sequence; the rest is padding
  const int64_t v0 = cu ? min(max((int64_t)cu[0], (int64_t)0), T) : 0;
  const int64_t v1 = cu ? min(max((int64_t)cu[nseq], v0), T) : T;
  const int64_t t = (int64_t)blockIdx.x * 1024 + threadIdx.x;
  const RowFlags f = row_flags(tokens, mask, t, T, V, select_all, v0, v1, sel_mask);
  int a = f.sel, k = f.keep;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { a += __shfl_xor(a, o, 64); k += __shfl_xor(k, o, 64); }
  if ((threadIdx.x & 63) == 0) { ws_sel[threadIdx.x >> 6] = a; ws_keep[threadIdx.x >> 6] = k; }
  __syncthreads();
  if (threadIdx.x == 0) {
    int sa = 0, sk = 0;
    for (int i = 0; i < 16; ++i) { sa += ws_sel[i]; sk += ws_keep[i]; }
    blk_counts[2 * blockIdx.x] = sa;
    blk_counts[2 * blockIdx.x + 1] = sk;
  }
}

__global__ __launch_bounds__(1024) void plan_write_kernel(const int32_t* __restrict__ tokens,
                                                          const uint8_t* __restrict__ mask, int64_t T, int V,
                                                          int select_all, float* __restrict__ scal,
                                                          int* __restrict__ cnt, int32_t* __restrict__ kept_idx,
                                                          int32_t* __restrict__ row_pos,
                                                          const int* __restrict__ cu, int nseq, int max_len,
                                                          uint8_t* __restrict__ mask_eff, int* __restrict__ status,
                                                          const int* __restrict__ blk_counts,
                                                          const uint8_t* __restrict__ sel_mask) {
  __shared__ int red_sel[16], red_keep[16], wave_sel[16];
  __shared__ int bad_cu;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nb = gridDim.x, b = blockIdx.x;
  const int64_t v0 = cu ? min(max((int64_t)cu[0], (int64_t)0), T) : 0;
  const int64_t v1 = cu ? min(max((int64_t)cu[nseq], v0), T) : T;
  // the offsets live on the device: block 0 checks them and reports through the status word (bit 1)
  if (b == 0) {
    if (tid == 0) bad_cu = 0;
    __syncthreads();
    if (cu) {
      int bad = 0;
      for (int i = tid; i <= nseq; i += 1024) {
        const int c = cu[i];
        if (c < 0 || c > T) bad = 1;
        if (i < nseq) {
          const int n = cu[i + 1] - c;
          if (n < 0 || n > max_len) bad = 1;
        }
      }
      if (bad) bad_cu = 1;   // benign race: every writer stores 1
    }
    __syncthreads();
    if (tid == 0) *status = bad_cu ? kStatusBadSeqlens : 0;
  }
  // selected / kept rows in the blocks before this one (fixed order of addition: integers, exact)
  int ps = 0, pk = 0;
  for (int i = tid; i < b; i += 1024) { ps += blk_counts[2 * i]; pk += blk_counts[2 * i + 1]; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { ps += __shfl_xor(ps, o, 64); pk += __shfl_xor(pk, o, 64); }
  if (lane == 0) { red_sel[w] = ps; red_keep[w] = pk; }
  const int64_t t = (int64_t)b * 1024 + tid;
  const RowFlags f = row_flags(tokens, mask, t, T, V, select_all, v0, v1, sel_mask);
  int incl = f.sel;   // inclusive scan inside the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wave_sel[w] = incl;
  __syncthreads();
  int base = 0, base_keep = 0, before = 0;
  for (int i = 0; i < 16; ++i) {
    base += red_sel[i];
    base_keep += red_keep[i];
    if (i < w) before += wave_sel[i];
  }
  if (t < T) {
    mask_eff[t] = (uint8_t)f.keep;
    if (f.sel) {
      const int pos = base + before + incl - 1;
      kept_idx[pos] = (int32_t)t;
      row_pos[t] = pos;
    } else {
      row_pos[t] = -1;
    }
  }
  if (b == nb - 1 && tid == 0) {
    const int total_sel = base + blk_counts[2 * b], total_keep = base_keep + blk_counts[2 * b + 1];
    const float n = fmaxf((float)total_keep, 1.f);
    scal[0] = n;
    scal[1] = 1.f / n;
    cnt[0] = total_sel;
  }
}

static inline int64_t plan_blocks(int64_t T) { return T > 0 ? (T + 1023) / 1024 : 1; }
size_t plan_rows_scratch_bytes(int64_t T) { return (size_t)plan_blocks(T) * 2 * sizeof(int); }

hipError_t launch_plan_rows(const int32_t* tokens, const uint8_t* mask, int64_t T, int V, int select_all,
                            float* scal, int* cnt, int32_t* kept_idx, int32_t* row_pos, const int* cu, int nseq,
                            int max_len, uint8_t* mask_eff, int* status, int* blk_counts, const uint8_t* sel_mask,
                            hipStream_t s) {
  ProfScope ps("plan_rows", 0, 24.0 * (double)T, s);
  const unsigned nb = (unsigned)plan_blocks(T);
  hipLaunchKernelGGL(plan_count_kernel, dim3(nb), dim3(1024), 0, s, tokens, mask, T, V, select_all, cu, nseq, blk_counts, sel_mask);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(plan_write_kernel, dim3(nb), dim3(1024), 0, s, tokens, mask, T, V, select_all, scal, cnt, kept_idx, row_pos, cu, nseq, max_len, mask_eff, status, blk_counts, sel_mask);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// Packed batches: position of every row inside its sequence (for RoPE), 0 for padding rows; and a fill
// that zeroes the rows no sequence owns (attention writes only rows of sequences, and everything that is
// later contracted over all T rows must be finite there).
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void seq_pos_kernel(const int* __restrict__ cu, int nseq, int64_t T, int max_len,
                                                      int32_t* __restrict__ pos) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  int p = 0;
  if (t >= cu[0] && t < cu[nseq]) {
    int lo = 0, hi = nseq;               // largest b with cu[b] <= t (empty sequences share offsets: any owner gives the same start)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    p = (int)(t - cu[lo]);
  }
  pos[t] = min(max(p, 0), max_len - 1);   // inside the RoPE table whatever the offsets hold
}

hipError_t launch_seq_pos(const int* cu, int nseq, int64_t T, int max_len, int32_t* pos, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipLaunchKernelGGL(seq_pos_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s, cu, nseq, T, max_len, pos);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void zero_padding_rows_kernel(uint32_t* __restrict__ p, const int* __restrict__ cu, int nseq,
                                                                int64_t T, int64_t row_words) {
  const int64_t t = blockIdx.x;
  if (t >= cu[0] && t < cu[nseq]) return;
  uint32_t* r = p + t * row_words;
  for (int64_t c = threadIdx.x; c < row_words; c += 256) r[c] = 0u;
}

// rows outside [cu[0], cu[nseq]) of a [T, row_bytes] array (row_bytes % 4 == 0) become zero
hipError_t launch_zero_padding_rows(void* p, const int* cu, int nseq, int64_t T, int64_t row_bytes, hipStream_t s) {
  if (T <= 0 || row_bytes <= 0) return hipSuccess;
  if (row_bytes % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(zero_padding_rows_kernel, dim3((unsigned)T), dim3(256), 0, s, (uint32_t*)p, cu, nseq, T, row_bytes / 4);
  return hipGetLastError();
}

// Row compaction.  Everything after the attention (output projection, MLP, final norm, LM head) is only
// needed for the rows the LM head processes: a row without loss influences the result through its key and
// value alone.  gather copies those rows (kept_idx, ascending) of up to two arrays into dense arrays and
// compacts labels and mask alongside; scatter is the inverse for gradients, writing zeros to the rows that
// were not selected.  The number of selected rows lives on the device.
template <typename T>
__device__ __forceinline__ void copy_row(const T* a, T* b, int d) {
  if ((d & 7) == 0) {
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      float v[8];
      ld8(a, c, v);
      st8(b, c, v);
    }
  } else {
    for (int c = threadIdx.x; c < d; c += 256) b[c] = a[c];
  }
}

template <typename T>
__device__ __forceinline__ void zero_row(T* b, int d) {
  if ((d & 7) == 0) {
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) st8(b, c, v);
  } else {
    for (int c = threadIdx.x; c < d; c += 256) stf(b, c, 0.f);
  }
}

// Embedding lookup of the token-input variant: one block per position.
template <typename T>
__global__ __launch_bounds__(256) void embed_rows_kernel(const T* __restrict__ embed, int rows,
                                                         const int32_t* __restrict__ ids, T* __restrict__ out, int d) {
  const size_t t = blockIdx.x;
  const int id = ids[t];
  T* b = out + t * (size_t)d;
  if (id >= 0 && id < rows) copy_row(embed + (size_t)id * (size_t)d, b, d);
  else zero_row(b, d);
}

hipError_t launch_embed_rows(int64_t T, int d, const void* embed, int rows, const int32_t* ids, void* out, int dtype,
                             hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps("embed_rows", 0, 2.0 * (double)T * d * dtype_size(dtype), s);
  dim3 grid((unsigned)T), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(embed_rows_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)embed, rows, ids, (bf16_t*)out, d);
  else hipLaunchKernelGGL(embed_rows_kernel<float>, grid, blk, 0, s, (const float*)embed, rows, ids, (float*)out, d);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T* __restrict__ src0, T* __restrict__ dst0, int d0,
                                                          const T* __restrict__ src1, T* __restrict__ dst1, int d1,
                                                          const int32_t* __restrict__ tokens,
                                                          const uint8_t* __restrict__ mask,
                                                          const int32_t* __restrict__ kept_idx,
                                                          const int* __restrict__ cnt,
                                                          int32_t* __restrict__ tokens_c, uint8_t* __restrict__ mask_c) {
  const int i = blockIdx.x;
  if (i >= *cnt) return;
  const size_t r = (size_t)kept_idx[i];
  copy_row(src0 + r * (size_t)d0, dst0 + (size_t)i * (size_t)d0, d0);
  if (src1) copy_row(src1 + r * (size_t)d1, dst1 + (size_t)i * (size_t)d1, d1);
  if (threadIdx.x == 0) {
    tokens_c[i] = tokens[r];
    mask_c[i] = mask[r];
  }
}

hipError_t launch_gather_rows(int64_t T, int d0, const void* src0, void* dst0, int d1, const void* src1, void* dst1,
                              const int32_t* tokens, const uint8_t* mask, const int32_t* kept_idx, const int* cnt,
                              int32_t* tokens_c, uint8_t* mask_c, int dtype, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps("gather_rows", 0, 2.0 * (double)T * (d0 + (src1 ? d1 : 0)) * dtype_size(dtype), s);
  prof_dynamic(cnt, 0, T);
  dim3 grid((unsigned)T), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(gather_rows_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)src0, (bf16_t*)dst0, d0, (const bf16_t*)src1, (bf16_t*)dst1, d1, tokens, mask, kept_idx, cnt, tokens_c, mask_c);
  else hipLaunchKernelGGL(gather_rows_kernel<float>, grid, blk, 0, s, (const float*)src0, (float*)dst0, d0, (const float*)src1, (float*)dst1, d1, tokens, mask, kept_idx, cnt, tokens_c, mask_c);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const T* __restrict__ src0, T* __restrict__ dst0, int d0,
                                                           const T* __restrict__ src1, T* __restrict__ dst1, int d1,
                                                           const int32_t* __restrict__ row_pos) {
  const size_t t = blockIdx.x;
  const int p = row_pos[t];
  if (p >= 0) {
    copy_row(src0 + (size_t)p * (size_t)d0, dst0 + t * (size_t)d0, d0);
    if (src1) copy_row(src1 + (size_t)p * (size_t)d1, dst1 + t * (size_t)d1, d1);
  } else {
    zero_row(dst0 + t * (size_t)d0, d0);
    if (src1) zero_row(dst1 + t * (size_t)d1, d1);
  }
}

hipError_t launch_scatter_rows(int64_t T, int d0, const void* src0, void* dst0, int d1, const void* src1, void* dst1,
                               const int32_t* row_pos, int dtype, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  ProfScope ps("scatter_rows", 0, 2.0 * (double)T * (d0 + (src1 ? d1 : 0)) * dtype_size(dtype), s);
  dim3 grid((unsigned)T), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(scatter_rows_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)src0, (bf16_t*)dst0, d0, (const bf16_t*)src1, (bf16_t*)dst1, d1, row_pos);
  else hipLaunchKernelGGL(scatter_rows_kernel<float>, grid, blk, 0, s, (const float*)src0, (float*)dst0, d0, (const float*)src1, (float*)dst1, d1, row_pos);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// RMSNorm forward: one 256-thread block per row.
// ----------------------------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T* __restrict__ x,
                                                          const T* __restrict__ g, float eps,
                                                          T* __restrict__ y, float* __restrict__ rstd,
                                                          int d, const int* __restrict__ rows_dev) {
  __shared__ float red[32];
  const size_t row = blockIdx.x;
  if (rows_dev && (int64_t)row >= (int64_t)*rows_dev) return;   // whole block, before any barrier
  const T* xr = x + row * (size_t)d;
  T* yr = y + row * (size_t)d;
  float ss = 0.f;
  if (VEC) {
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      float v[8];
      ld8(xr, c, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
    }
  } else {
    for (int c = threadIdx.x; c < d; c += 256) {
      float v = ldf(xr, c);
      ss += v * v;
    }
  }
  float tot = block_sum(ss, red);
  float r = 1.0f / sqrtf(tot / (float)d + eps);
  if (threadIdx.x == 0) rstd[row] = r;
  if (VEC) {
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
      float v[8], gg[8], o[8];
      ld8(xr, c, v);
      ld8(g, c, gg);
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = gg[j] * v[j] * r;
      st8(yr, c, o);
    }
  } else {
    for (int c = threadIdx.x; c < d; c += 256) stf(yr, c, ldf(g, c) * ldf(xr, c) * r);
  }
}

hipError_t launch_rmsnorm_fwd(int64_t rows, int d, const void* x, const void* g, float eps, void* y,
                              float* rstd, int dtype, const int* rows_dev, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  ProfScope ps("rmsnorm_fwd", 0, (double)rows * d * 2.0 * dtype_size(dtype) + 4.0 * rows, s);
  if (rows_dev) prof_dynamic(rows_dev, 0, rows);
  dim3 grid((unsigned)rows), blk(256);
  const bool vec = (d % 8) == 0;
  if (dtype == kBF16) {
    if (vec) hipLaunchKernelGGL((rmsnorm_fwd_kernel<bf16_t, true>), grid, blk, 0, s, (const bf16_t*)x, (const bf16_t*)g, eps, (bf16_t*)y, rstd, d, rows_dev);
    else hipLaunchKernelGGL((rmsnorm_fwd_kernel<bf16_t, false>), grid, blk, 0, s, (const bf16_t*)x, (const bf16_t*)g, eps, (bf16_t*)y, rstd, d, rows_dev);
  } else {
    if (vec) hipLaunchKernelGGL((rmsnorm_fwd_kernel<float, true>), grid, blk, 0, s, (const float*)x, (const float*)g, eps, (float*)y, rstd, d, rows_dev);
    else hipLaunchKernelGGL((rmsnorm_fwd_kernel<float, false>), grid, blk, 0, s, (const float*)x, (const float*)g, eps, (float*)y, rstd, d, rows_dev);
  }
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// RMSNorm backward.  u = g*dy; dx = r*u - x*r^3*<u,x>/d (+ residual gradient);
// dg[c] = sum_rows dy*x*r, reduced in two stages: each block owns a contiguous share of the rows and keeps its
// column partials in registers, then a column-sum kernel folds the per-block partials.
// Vector path: d % 8 == 0 and d <= 8192.  Scalar path: d <= 1024.
// ----------------------------------------------------------------------------------------------
// The grid is what the chip holds at once (256 CUs x blocks per CU at the kernel's register count), at
// least kMinRowsPerBlock rows each, and the rows are split evenly over it: one round, no partly filled second.
constexpr int kMinRowsPerBlock = 8;
__host__ __device__ inline int rmsnorm_bwd_nit(int d) {
  const bool vec = (d % 8) == 0 && d <= 8192;
  const int per = vec ? 8 * 256 : 256;   // columns covered by one pass of the block
  return (d + per - 1) / per;
}
inline int64_t rmsnorm_bwd_blocks(int64_t rows, int d) {
  const int nit = rmsnorm_bwd_nit(d);
  const int64_t cap = 256 * (nit <= 1 ? 5 : nit == 2 ? 3 : 2);
  const int64_t want = (rows + kMinRowsPerBlock - 1) / kMinRowsPerBlock;
  return want < 1 ? 1 : (want < cap ? want : cap);
}

template <typename T, bool VEC, int NIT>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ dy,
                                                          const T* __restrict__ x,
                                                          const T* __restrict__ g,
                                                          const float* __restrict__ rstd,
                                                          const T* __restrict__ res, T* __restrict__ dx,
                                                          float* __restrict__ dg_partial, int64_t rows,
                                                          int d, const int* __restrict__ rows_dev) {
  __shared__ float red[32];
  if (rows_dev) rows = min(rows, (int64_t)max(*rows_dev, 0));   // blocks past the end write zero partials
  constexpr int W = VEC ? 8 : 1;   // a thread owns NIT groups of W columns
  float acc[NIT][W];
#pragma unroll
  for (int it = 0; it < NIT; ++it)
#pragma unroll
    for (int j = 0; j < W; ++j) acc[it][j] = 0.f;

  const int64_t per_block = (rows + (int64_t)gridDim.x - 1) / (int64_t)gridDim.x;
  const int64_t r0 = min(rows, (int64_t)blockIdx.x * per_block);
  const int64_t r1 = min(rows, r0 + per_block);
  const float inv_d = 1.0f / (float)d;
  float gg[NIT][W];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = (threadIdx.x + it * 256) * W;
#pragma unroll
    for (int j = 0; j < W; ++j) gg[it][j] = 0.f;
    if (c < d) {
      if constexpr (VEC) ld8(g, c, gg[it]);
      else gg[it][0] = ldf(g, c);
    }
  }
  // The rows of a block are walked with a one-row look-ahead: the loads of row+1 are issued before the
  // block-wide reduction of row, whose two barriers would otherwise expose the full memory latency per row.
  // Two things keep those loads in flight: they are held as loaded (no conversion, which would need the
  // value at once) until the next iteration, and the reduction uses barriers that order LDS only.
  struct RowRaw {
    Raw8<T> x[NIT], dy[NIT], res[NIT];   // vector path
    float xs[NIT], dys[NIT], ress[NIT];  // scalar path
    float rstd;
  } nxt;
  auto load_row = [&](int64_t row) {
    const size_t base = (size_t)row * (size_t)d;
    nxt.rstd = rstd[row];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (threadIdx.x + it * 256) * W;
      if constexpr (VEC) {
        nxt.x[it].zero(); nxt.dy[it].zero(); nxt.res[it].zero();
        if (c < d) {
          nxt.dy[it].load(dy, base + c);
          nxt.x[it].load(x, base + c);
          if (res) nxt.res[it].load(res, base + c);
        }
      } else {
        nxt.xs[it] = nxt.dys[it] = nxt.ress[it] = 0.f;
        if (c < d) {
          nxt.dys[it] = ldf(dy, base + c);
          nxt.xs[it] = ldf(x, base + c);
          if (res) nxt.ress[it] = ldf(res, base + c);
        }
      }
    }
  };
  if (r0 < r1) load_row(r0);
  for (int64_t row = r0; row < r1; ++row) {
    const size_t base = (size_t)row * (size_t)d;
    const float r = nxt.rstd;
    float xv[NIT][W], dyv[NIT][W], rv[NIT][W];
    float dot = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if constexpr (VEC) {
        nxt.x[it].get(xv[it]); nxt.dy[it].get(dyv[it]); nxt.res[it].get(rv[it]);
      } else {
        xv[it][0] = nxt.xs[it]; dyv[it][0] = nxt.dys[it]; rv[it][0] = nxt.ress[it];
      }
#pragma unroll
      for (int j = 0; j < W; ++j) dot += gg[it][j] * dyv[it][j] * xv[it][j];
    }
    if (row + 1 < r1) load_row(row + 1);
    const float tot = block_sum_lds(dot, red);   // LDS-only barriers: the loads just issued stay in flight
    const float coef = r * r * r * tot * inv_d;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (threadIdx.x + it * 256) * W;
      if (c < d) {
        float o[W];
#pragma unroll
        for (int j = 0; j < W; ++j) {
          o[j] = rv[it][j] + (r * (gg[it][j] * dyv[it][j]) - xv[it][j] * coef);
          acc[it][j] += dyv[it][j] * xv[it][j] * r;
        }
        if constexpr (VEC) st8(dx, base + c, o);
        else stf(dx, base + c, o[0]);
      }
    }
  }
  float* out = dg_partial + (size_t)blockIdx.x * (size_t)d;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = (threadIdx.x + it * 256) * W;
    if (c < d) {
#pragma unroll
      for (int j = 0; j < W; ++j) out[c + j] = acc[it][j];
    }
  }
}

// out[c] = sum_r part[r, c]; 16 columns x 16 row lanes per block, four loads in flight per thread, fixed
// summation order.  (64 columns x 4 row lanes, i.e. 64 blocks at d = 4096 with one load in flight per thread, took
// 49 us for the 768 x 4096 partials of the 8B shape: a fifth of the RMSNorm backward it finishes.)
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ part, int64_t nrows, int d,
                                                     float* __restrict__ out, int accumulate) {
  __shared__ float sm[16][17];
  const int cl = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (c < d) {
    int64_t r = rl;
    for (; r + 48 < nrows; r += 64) {
      a0 += part[(size_t)r * d + c];
      a1 += part[(size_t)(r + 16) * d + c];
      a2 += part[(size_t)(r + 32) * d + c];
      a3 += part[(size_t)(r + 48) * d + c];
    }
    for (; r < nrows; r += 16) a0 += part[(size_t)r * d + c];
  }
  sm[rl][cl] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (rl == 0 && c < d) {
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) v += sm[i][cl];
    out[c] = accumulate ? out[c] + v : v;
  }
}

size_t rmsnorm_bwd_scratch_bytes(int64_t rows, int d) {
  const int64_t nblk = rmsnorm_bwd_blocks(rows, d);
  return (size_t)nblk * (size_t)d * sizeof(float);
}

hipError_t launch_rmsnorm_bwd(int64_t rows, int d, const void* dy, const void* x, const void* g,
                              const float* rstd, const void* res, void* dx, float* dg, float* dg_partial,
                              int dtype, const int* rows_dev, hipStream_t s, int accumulate) {
  if (rows <= 0) return hipSuccess;
  const bool vec = (d % 8) == 0 && d <= 8192;
  if (!vec && d > 1024) return hipErrorInvalidValue;
  ProfScope ps("rmsnorm_bwd", 0, (double)rows * d * (res ? 4.0 : 3.0) * dtype_size(dtype) + 4.0 * rows, s);
  if (rows_dev) prof_dynamic(rows_dev, 0, rows);
  const int64_t nblk = rmsnorm_bwd_blocks(rows, d);
  dim3 grid((unsigned)nblk), blk(256);
  const int per = vec ? 8 * 256 : 256;            // columns covered by one pass of the block
  const int nit = (d + per - 1) / per;            // <= 4 by the limits above
#define TIDE_RMS_BWD(T, V, N) hipLaunchKernelGGL((rmsnorm_bwd_kernel<T, V, N>), grid, blk, 0, s, (const T*)dy, (const T*)x, (const T*)g, rstd, (const T*)res, (T*)dx, dg_partial, rows, d, rows_dev)
#define TIDE_RMS_BWD_N(T, V) do { if (nit <= 1) TIDE_RMS_BWD(T, V, 1); else if (nit == 2) TIDE_RMS_BWD(T, V, 2); else TIDE_RMS_BWD(T, V, 4); } while (0)
  if (dtype == kBF16) {
    if (vec) TIDE_RMS_BWD_N(bf16_t, true); else TIDE_RMS_BWD_N(bf16_t, false);
  } else {
    if (vec) TIDE_RMS_BWD_N(float, true); else TIDE_RMS_BWD_N(float, false);
  }
#undef TIDE_RMS_BWD_N
#undef TIDE_RMS_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_kernel, dim3((d + 15) / 16), dim3(256), 0, s, dg_partial, nblk, d, dg, accumulate);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// RoPE.  The cos/sin table is built once per call in double precision (positions reach 16384, where
// an fp32 angle would already be off by ~1e-3 rad), then applied in place to the q and k heads.
// ----------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(int S, int half, int dh, double theta, float* __restrict__ cs) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= S * half) return;
  const int pos = idx / half, i = idx % half;
  const double inv = pow(theta, -2.0 * (double)i / (double)dh);
  const double ang = (double)pos * inv;
  cs[2 * (size_t)idx] = (float)cos(ang);
  cs[2 * (size_t)idx + 1] = (float)sin(ang);
}

hipError_t launch_rope_table(int S, int dh, float theta, float* cs, hipStream_t s) {
  const int half = dh / 2;
  const int n = S * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, S, half, dh, (double)theta, cs);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ qkv, const float* __restrict__ cs,
                                                   int S, int nrot_heads, int dh, int ld, float sgn,
                                                   int64_t total, const int32_t* __restrict__ row_pos, int pos_offset) {
  // one thread per (row t, head, i < dh/2); q heads then k heads are the first nrot_heads heads of a row
  const int half = dh >> 1;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int i = (int)(idx % half);
  const int64_t th = idx / half;
  const int hd = (int)(th % nrot_heads);
  const int64_t t = th / nrot_heads;
  const int pos = (row_pos ? row_pos[t] : (int)(t % S)) + pos_offset;
  const float c = cs[2 * ((size_t)pos * half + i)];
  const float sn = sgn * cs[2 * ((size_t)pos * half + i) + 1];
  const size_t o = (size_t)t * ld + (size_t)hd * dh + i;
  const float x1 = ldf(qkv, o), x2 = ldf(qkv, o + half);
  stf(qkv, o, x1 * c - x2 * sn);
  stf(qkv, o + half, x2 * c + x1 * sn);
}

// Eight pairs per thread (16-byte accesses); needs head_dim % 16 == 0 and a 16-byte aligned buffer.
template <typename T>
__global__ __launch_bounds__(256) void rope_vec8_kernel(T* __restrict__ qkv, const float* __restrict__ cs,
                                                        int S, int nrot_heads, int dh, int ld, float sgn,
                                                        int64_t total8, const int32_t* __restrict__ row_pos,
                                                        int pos_offset) {
  const int half = dh >> 1, h8 = half >> 3;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total8) return;
  const int i = (int)(idx % h8) * 8;
  const int64_t th = idx / h8;
  const int hd = (int)(th % nrot_heads);
  const int64_t t = th / nrot_heads;
  const int pos = (row_pos ? row_pos[t] : (int)(t % S)) + pos_offset;
  const float4* tab = reinterpret_cast<const float4*>(cs + 2 * ((size_t)pos * half + i));   // (cos, sin) x 8
  const size_t o = (size_t)t * ld + (size_t)hd * dh + i;
  float x1[8], x2[8], y1[8], y2[8];
  ld8(qkv, o, x1);
  ld8(qkv, o + half, x2);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float4 v = tab[j];
    const float c0 = v.x, s0 = sgn * v.y, c1 = v.z, s1 = sgn * v.w;
    y1[2 * j] = x1[2 * j] * c0 - x2[2 * j] * s0;
    y2[2 * j] = x2[2 * j] * c0 + x1[2 * j] * s0;
    y1[2 * j + 1] = x1[2 * j + 1] * c1 - x2[2 * j + 1] * s1;
    y2[2 * j + 1] = x2[2 * j + 1] * c1 + x1[2 * j + 1] * s1;
  }
  st8(qkv, o, y1);
  st8(qkv, o + half, y2);
}

hipError_t launch_rope(int B, int S, int nh, int nkv, int dh, const float* cs, void* qkv, int inverse,
                       int dtype, const int32_t* row_pos, int pos_offset, hipStream_t s) {
  const int nrot = nh + nkv;
  const int ld = (nh + 2 * nkv) * dh;
  const int64_t total = (int64_t)B * S * nrot * (dh / 2);
  if (total <= 0) return hipSuccess;
  const float sgn = inverse ? -1.f : 1.f;
  ProfScope ps("rope", 0, (double)total * 4.0 * dtype_size(dtype), s);
  if ((dh % 16) == 0 && (((uintptr_t)qkv | (uintptr_t)cs) & 15) == 0) {
    const int64_t total8 = total / 8;
    dim3 grid8((unsigned)((total8 + 255) / 256)), blk8(256);
    if (dtype == kBF16) hipLaunchKernelGGL(rope_vec8_kernel<bf16_t>, grid8, blk8, 0, s, (bf16_t*)qkv, cs, S, nrot, dh, ld, sgn, total8, row_pos, pos_offset);
    else hipLaunchKernelGGL(rope_vec8_kernel<float>, grid8, blk8, 0, s, (float*)qkv, cs, S, nrot, dh, ld, sgn, total8, row_pos, pos_offset);
    return hipGetLastError();
  }
  dim3 grid((unsigned)((total + 255) / 256)), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(rope_kernel<bf16_t>, grid, blk, 0, s, (bf16_t*)qkv, cs, S, nrot, dh, ld, sgn, total, row_pos, pos_offset);
  else hipLaunchKernelGGL(rope_kernel<float>, grid, blk, 0, s, (float*)qkv, cs, S, nrot, dh, ld, sgn, total, row_pos, pos_offset);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// SwiGLU
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }

template <typename T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const T* __restrict__ gt, const T* __restrict__ u,
                                                         T* __restrict__ h, int64_t n, int64_t per_row,
                                                         const int* __restrict__ rows_dev) {
  if (rows_dev) n = min(n, (int64_t)max(*rows_dev, 0) * per_row);
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i0 + 8 <= n) {
    float a[8], b[8], o[8];
    ld8(gt, i0, a);
    ld8(u, i0, b);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = a[j] * sigmoidf_(a[j]) * b[j];
    st8(h, i0, o);
  } else {
    for (int64_t i = i0; i < n; ++i) {
      float a = ldf(gt, i);
      stf(h, i, a * sigmoidf_(a) * ldf(u, i));
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T* __restrict__ dh, const T* gt, const T* u,
                                                         T* dgt, T* du, int64_t n, int64_t per_row,
                                                         const int* __restrict__ rows_dev) {
  // dgt/du may alias gt/u: every element is read before it is written by the same thread
  if (rows_dev) n = min(n, (int64_t)max(*rows_dev, 0) * per_row);
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i0 + 8 <= n) {
    float a[8], b[8], c[8], o1[8], o2[8];
    ld8(gt, i0, a);
    ld8(u, i0, b);
    ld8(dh, i0, c);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float sg = sigmoidf_(a[j]);
      o1[j] = c[j] * b[j] * sg * (1.f + a[j] * (1.f - sg));
      o2[j] = c[j] * a[j] * sg;
    }
    st8(dgt, i0, o1);
    st8(du, i0, o2);
  } else {
    for (int64_t i = i0; i < n; ++i) {
      float a = ldf(gt, i), b = ldf(u, i), c = ldf(dh, i);
      float sg = sigmoidf_(a);
      stf(dgt, i, c * b * sg * (1.f + a * (1.f - sg)));
      stf(du, i, c * a * sg);
    }
  }
}

// n = rows * per_row elements; with rows_dev only the first *rows_dev rows are touched
hipError_t launch_swiglu_fwd(int64_t n, const void* gt, const void* u, void* h, int dtype, int64_t per_row,
                             const int* rows_dev, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (rows_dev && (per_row <= 0 || n % per_row)) return hipErrorInvalidValue;
  ProfScope ps("swiglu_fwd", 0, (double)n * 3.0 * dtype_size(dtype), s);
  if (rows_dev) prof_dynamic(rows_dev, 0, n / per_row);
  dim3 grid((unsigned)((n + 2047) / 2048)), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(swiglu_fwd_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)gt, (const bf16_t*)u, (bf16_t*)h, n, per_row, rows_dev);
  else hipLaunchKernelGGL(swiglu_fwd_kernel<float>, grid, blk, 0, s, (const float*)gt, (const float*)u, (float*)h, n, per_row, rows_dev);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd(int64_t n, const void* dh, const void* gt, const void* u, void* dgt, void* du,
                             int dtype, int64_t per_row, const int* rows_dev, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (rows_dev && (per_row <= 0 || n % per_row)) return hipErrorInvalidValue;
  ProfScope ps("swiglu_bwd", 0, (double)n * 5.0 * dtype_size(dtype), s);
  if (rows_dev) prof_dynamic(rows_dev, 0, n / per_row);
  dim3 grid((unsigned)((n + 2047) / 2048)), blk(256);
  if (dtype == kBF16) hipLaunchKernelGGL(swiglu_bwd_kernel<bf16_t>, grid, blk, 0, s, (const bf16_t*)dh, (const bf16_t*)gt, (const bf16_t*)u, (bf16_t*)dgt, (bf16_t*)du, n, per_row, rows_dev);
  else hipLaunchKernelGGL(swiglu_bwd_kernel<float>, grid, blk, 0, s, (const float*)dh, (const float*)gt, (const float*)u, (float*)dgt, (float*)du, n, per_row, rows_dev);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// Cross-entropy over a block of logits z [rows, ldz] (ldz % 8 == 0, rows 16-byte aligned).
// Statistics: one block per row, online (max, sum-exp) per thread, then a block combine.
// ----------------------------------------------------------------------------------------------
template <typename T, bool TOP1>
__global__ __launch_bounds__(256) void ce_stats_kernel(const T* __restrict__ z, int64_t ldz, int V,
                                                       const int32_t* __restrict__ tokens,
                                                       const uint8_t* __restrict__ mask,
                                                       float* __restrict__ lse,
                                                       float* __restrict__ loss_rows,
                                                       int32_t* __restrict__ top1,
                                                       const int32_t* __restrict__ top1_idx,
                                                       float* __restrict__ hit_rows,
                                                       const int* __restrict__ rows_dev, int rows_off) {
  __shared__ float sm_m[4], sm_s[4], sm_bv[4];
  __shared__ int sm_bi[4];
  const size_t row = blockIdx.x;
  if (rows_dev && (int)row >= *rows_dev - rows_off) return;
  const T* zr = z + row * (size_t)ldz;
  float m = -INFINITY, ssum = 0.f;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int c = threadIdx.x * 8; c < V; c += 256 * 8) {
    float v[8];
    if (c + 8 <= V) {
      ld8(zr, c, v);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (c + j < V) ? ldf(zr, c + j) : -INFINITY;
    }
    float cm = v[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) cm = fmaxf(cm, v[j]);
    if (TOP1) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (v[j] > bv) { bv = v[j]; bi = c + j; }  // ascending c: first maximum is kept
    }
    const float nm = fmaxf(m, cm);
    float part = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) part += __expf(v[j] - nm);
    ssum = ssum * __expf(m - nm) + part;
    m = nm;
  }
  // wave combine
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float om = __shfl_xor(m, o, 64), os = __shfl_xor(ssum, o, 64);
    float nm = fmaxf(m, om);
    float sa = (m == -INFINITY) ? 0.f : ssum * __expf(m - nm);
    float sb = (om == -INFINITY) ? 0.f : os * __expf(om - nm);
    ssum = sa + sb;
    m = nm;
    if (TOP1) {
      float obv = __shfl_xor(bv, o, 64);
      int obi = __shfl_xor(bi, o, 64);
      if (obv > bv || (obv == bv && obi < bi)) { bv = obv; bi = obi; }
    }
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    sm_m[w] = m; sm_s[w] = ssum; sm_bv[w] = bv; sm_bi[w] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm_m[0], Sx = sm_s[0], BV = sm_bv[0];
    int BI = sm_bi[0];
    for (int i = 1; i < 4; ++i) {
      float om = sm_m[i], os = sm_s[i];
      float nm = fmaxf(M, om);
      float sa = (M == -INFINITY) ? 0.f : Sx * __expf(M - nm);
      float sb = (om == -INFINITY) ? 0.f : os * __expf(om - nm);
      Sx = sa + sb;
      M = nm;
      if (sm_bv[i] > BV || (sm_bv[i] == BV && sm_bi[i] < BI)) { BV = sm_bv[i]; BI = sm_bi[i]; }
    }
    const float l = M + logf(Sx);
    lse[row] = l;
    const int tk = tokens[row];
    const bool keep = mask[row] != 0 && tk >= 0 && tk < V;
    loss_rows[row] = keep ? (l - ldf(zr, (size_t)tk)) : 0.f;
    if (TOP1) {
      if (top1) top1[top1_idx ? top1_idx[row] : (int)row] = BI;
      if (hit_rows) hit_rows[row] = (keep && BI == tk) ? 1.f : 0.f;
    }
  }
}

hipError_t launch_ce_stats(int64_t rows, int V, const void* z, int64_t ldz, const int32_t* tokens,
                           const uint8_t* mask, float* lse, float* loss_rows, int32_t* top1,
                           const int32_t* top1_idx, float* hit_rows, const int* rows_dev, int64_t rows_off,
                           int dtype, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (ldz % 8 != 0) return hipErrorInvalidValue;
  ProfScope ps("ce_stats", 0, (double)rows * V * dtype_size(dtype), s);
  if (rows_dev) prof_dynamic(rows_dev, rows_off, rows);
  dim3 grid((unsigned)rows), blk(256);
  const int ro = (int)rows_off;
  if (dtype == kBF16) {
    if (top1 || hit_rows) hipLaunchKernelGGL((ce_stats_kernel<bf16_t, true>), grid, blk, 0, s, (const bf16_t*)z, ldz, V, tokens, mask, lse, loss_rows, top1, top1_idx, hit_rows, rows_dev, ro);
    else hipLaunchKernelGGL((ce_stats_kernel<bf16_t, false>), grid, blk, 0, s, (const bf16_t*)z, ldz, V, tokens, mask, lse, loss_rows, top1, top1_idx, hit_rows, rows_dev, ro);
  } else {
    if (top1 || hit_rows) hipLaunchKernelGGL((ce_stats_kernel<float, true>), grid, blk, 0, s, (const float*)z, ldz, V, tokens, mask, lse, loss_rows, top1, top1_idx, hit_rows, rows_dev, ro);
    else hipLaunchKernelGGL((ce_stats_kernel<float, false>), grid, blk, 0, s, (const float*)z, ldz, V, tokens, mask, lse, loss_rows, top1, top1_idx, hit_rows, rows_dev, ro);
  }
  return hipGetLastError();
}

// Training pass over a block of logits with the statistics and the gradient in ONE kernel: a block owns a
// row, reads it for the online (max, sum-exp), and reads it again to write dz over it.  The second read of
// the 250 KB row comes out of the memory-side cache instead of HBM as long as few enough rows are in
// flight: 48 KB of unused dynamic LDS per block hold that to three 512-thread blocks per CU (measured: 3.42 ms
// against 3.75 ms for two separate kernels at the 8B shape; 3.9 ms with four blocks per CU, 3.7 with two).
// Outputs: lse, the row's loss term keep * (lse - z[label]), and dz = keep * (exp(z - lse) - onehot(label))
// written over z, unscaled by 1/N; columns in [V, ldz) are zeroed so that the padded tail never contributes
// to the products that read dz with K = V rounded up.
template <typename T>
__global__ __launch_bounds__(512) void ce_train_kernel(T* __restrict__ z, int64_t ldz, int V,
                                                       const int32_t* __restrict__ tokens,
                                                       const uint8_t* __restrict__ mask, float* __restrict__ lse,
                                                       float* __restrict__ loss_rows,
                                                       const int* __restrict__ rows_dev, int rows_off) {
  __shared__ float sm_m[8], sm_s[8];
  __shared__ float sm_l;
  const size_t row = blockIdx.x;
  if (rows_dev && (int)row >= *rows_dev - rows_off) return;   // whole block, before any barrier
  T* zr = z + row * (size_t)ldz;
  const int tk = tokens[row];
  const bool keep = mask[row] != 0 && tk >= 0 && tk < V;
  float m = -INFINITY, ssum = 0.f;
  for (int c = threadIdx.x * 8; c < V; c += 512 * 8) {
    float v[8];
    if (c + 8 <= V) {
      ld8(zr, c, v);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (c + j < V) ? ldf(zr, c + j) : -INFINITY;
    }
    float cm = v[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) cm = fmaxf(cm, v[j]);
    const float nm = fmaxf(m, cm);
    float part = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) part += __expf(v[j] - nm);
    ssum = ssum * __expf(m - nm) + part;
    m = nm;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o, 64), os = __shfl_xor(ssum, o, 64);
    const float nm = fmaxf(m, om);
    const float sa = (m == -INFINITY) ? 0.f : ssum * __expf(m - nm);
    const float sb = (om == -INFINITY) ? 0.f : os * __expf(om - nm);
    ssum = sa + sb;
    m = nm;
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sm_m[w] = m; sm_s[w] = ssum; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm_m[0], Sx = sm_s[0];
    for (int i = 1; i < 8; ++i) {
      const float om = sm_m[i], os = sm_s[i];
      const float nm = fmaxf(M, om);
      const float sa = (M == -INFINITY) ? 0.f : Sx * __expf(M - nm);
      const float sb = (om == -INFINITY) ? 0.f : os * __expf(om - nm);
      Sx = sa + sb;
      M = nm;
    }
    const float l = M + logf(Sx);
    lse[row] = l;
    loss_rows[row] = keep ? (l - ldf(zr, (size_t)tk)) : 0.f;   // before anything of the row is overwritten
    sm_l = l;
  }
  __syncthreads();
  const float l = sm_l;
  for (int c = threadIdx.x * 8; c < ldz; c += 512 * 8) {
    float v[8], o[8];
    ld8(zr, c, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float p = __expf(v[j] - l) - ((c + j == tk) ? 1.f : 0.f);
      o[j] = (keep && (c + j < V)) ? p : 0.f;
    }
    st8(zr, c, o);
  }
}

// The same pass for bf16 logits with the ROW HELD ON THE CU between the statistics and the gradient, so that it
// is read from memory once and written once (2 x 7.1 GB instead of 3 x at the 8B shape).  A block of 512 threads
// owns a row; thread t keeps the 16-byte chunks t, t + 512, ...: the first NREG of them in registers, the other
// n_lds in LDS (its own slots: no sharing).  NREG is chosen by the launcher so that every register chunk lies
// wholly below V: only LDS chunks can hold padded columns or lie past the row, and they are cleaned on their way
// into LDS.  At 128256 columns that is 24 chunks in registers + 8 in LDS = 64 KiB per block, so TWO blocks fit a
// CU and the arithmetic of one overlaps the loads and stores of the other (the whole row in the registers of one
// 1024-thread block measured 5.5 ms against 3.4 ms for the two-read kernel: the pass needs some 15 vector
// instructions per element, as long per row as the memory traffic takes).
// The softmax is the exact two-step one: block maximum first, then one exponential per element for the sum and
// one for the gradient, each as exp2(fma(z, log2 e, -shift * log2 e)).  Same outputs as ce_train_kernel.
// cache policy bits of the row's loads and stores (0 = default, 2 = non-temporal).  Measured at the 8B shape:
// 2.75 ms with default policy on both, 2.68 with non-temporal loads, 2.65 with non-temporal stores, 2.59 with both
// (the two-read kernel in the same call: 3.41 ms).
#ifndef TIDE_CE_LOAD_AUX
#define TIDE_CE_LOAD_AUX 2
#endif
#ifndef TIDE_CE_STORE_AUX
#define TIDE_CE_STORE_AUX 2
#endif
template <int NREG>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
void ce_train_resident_kernel(bf16_t* __restrict__ z, int64_t ldz, int V, int n_lds,
                              const int32_t* __restrict__ tokens, const uint8_t* __restrict__ mask,
                              float* __restrict__ lse, float* __restrict__ loss_rows,
                              const int* __restrict__ rows_dev, int rows_off) {
  constexpr int NT = 512, STEP = NT * 8;                     // columns between two chunks of a thread
  constexpr float LOG2E = 1.4426950408889634f;
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  extern __shared__ u32x4_t ce_row_lds[];                      // n_lds x NT chunks
  __shared__ float sm_red[8];
  __shared__ float sm_bc[3];
  const size_t row = blockIdx.x;
  if (rows_dev && (int)row >= *rows_dev - rows_off) return;   // whole block, before any barrier
  bf16_t* zr = z + row * (size_t)ldz;
  const int tk = tokens[row];
  const bool keep = mask[row] != 0 && tk >= 0 && tk < V;
  const int c0 = threadIdx.x * 8;
  u32x4_t* mine_lds = ce_row_lds + threadIdx.x;
  // The row as a buffer resource: one 32-bit offset register per thread serves every chunk (the chunk's
  // distance is a scalar offset), and the hardware drops what lies past the row (loads give 0, stores vanish).
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(zr, 0, (int)((uint32_t)ldz * 2u), 0x00020000);
  const uint32_t off0 = (uint32_t)c0 * 2u;
  auto fetch = [&](uint32_t voff, int soff) {
    return __builtin_bit_cast(u32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, TIDE_CE_LOAD_AUX));
  };
  auto store = [&](u32x4_t v, uint32_t voff, int soff) { __builtin_amdgcn_raw_buffer_store_b128(v, rs, voff, soff, TIDE_CE_STORE_AUX); };
  const u32x4_t zero4 = {0u, 0u, 0u, 0u};
  u32x4_t buf[NREG > 0 ? NREG : 1];
  // all loads first, none of them conditional
#pragma unroll
  for (int i = 0; i < NREG; ++i) buf[i] = fetch(off0, i * STEP * 2);
  for (int i = 0; i < n_lds; ++i) {
    // columns >= V become -inf (bf16 0xFF80) in the packed chunk itself, so that no pass needs a column test
    // (the whole distance in the vector offset here: that is the part the range check surely covers)
    const int c = c0 + (NREG + i) * STEP;
    u32x4_t v = fetch((uint32_t)c * 2u, 0);
    const int nv = V - c;
    if (nv < 8) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        v[k] = (2 * k + 1 < nv) ? v[k] : (2 * k < nv) ? ((v[k] & 0xFFFFu) | 0xFF800000u) : 0xFF80FF80u;
    }
    mine_lds[i * NT] = v;
  }
  // the owner of the label's element: chunk and position (chunk -1: not in this thread)
  const int dl = tk - c0;
  const bool mine = keep && dl >= 0 && (dl & (STEP - 1)) < 8;
  const int sel_i = mine ? dl / STEP : -1, sel_j = dl & 7;
  // Every pass walks the register chunks strictly one after the other: a chunk is made opaque to the compiler
  // together with the pass's running value right before its turn, so neither the unpacked floats of a whole
  // pass nor those of an earlier pass are kept alive (8 registers per chunk instead of 4, and spills).
  auto turn = [&](int i, float& running) {
    asm volatile("" : "+v"(running), "+v"(buf[i]));
  };
  auto lo = [](uint32_t w) { return __uint_as_float(w << 16); };
  auto hi = [](uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); };
  auto max3 = [](float a, float b, float c) {                 // (plain fmaxf first quiets each unpacked operand)
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
  };
  auto chunk_max = [&](u32x4_t v, float m) {
#pragma unroll
    for (int k = 0; k < 4; ++k) m = max3(m, lo(v[k]), hi(v[k]));
    return m;
  };
  auto pick = [&](u32x4_t v) {                                // the label's logit (one thread of the block, once)
    const uint32_t w = sel_j < 2 ? v[0] : sel_j < 4 ? v[1] : sel_j < 6 ? v[2] : v[3];
    sm_bc[2] = (sel_j & 1) ? hi(w) : lo(w);
  };
  auto chunk_sum = [&](u32x4_t wv, float sh) {                // sum of exp2(z log2e + sh); exp2(-inf) = 0
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      part += __builtin_amdgcn_exp2f(fmaf(lo(wv[k]), LOG2E, sh)) + __builtin_amdgcn_exp2f(fmaf(hi(wv[k]), LOG2E, sh));
    return part;
  };
  auto chunk_grad = [&](u32x4_t wv, float sh, bool owner) {   // exp(z - lse), minus 1 at the label, packed
    u32x4_t pk;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      pk[k] = f2bf2(__builtin_amdgcn_exp2f(fmaf(lo(wv[k]), LOG2E, sh)), __builtin_amdgcn_exp2f(fmaf(hi(wv[k]), LOG2E, sh)));
    if (owner) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (sel_j == j) {
          const float e = (j & 1) ? hi(wv[j >> 1]) : lo(wv[j >> 1]);
          const uint32_t h = f2bf(__builtin_amdgcn_exp2f(fmaf(e, LOG2E, sh)) - 1.f);
          pk[j >> 1] = (j & 1) ? ((pk[j >> 1] & 0xFFFFu) | (h << 16)) : ((pk[j >> 1] & 0xFFFF0000u) | h);
        }
    }
    return pk;
  };

  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NREG; ++i) {
    turn(i, m);
    m = chunk_max(buf[i], m);
    if (sel_i == i) pick(buf[i]);
  }
  for (int i = 0; i < n_lds; ++i) {
    const u32x4_t v = mine_lds[i * NT];
    m = chunk_max(v, m);
    if (sel_i == NREG + i) pick(v);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sm_red[w] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm_red[0];
    for (int i = 1; i < 8; ++i) M = fmaxf(M, sm_red[i]);
    sm_bc[0] = M;
  }
  __syncthreads();
  const float M = sm_bc[0];
  const float nM = -M * LOG2E;
  float ssum = 0.f;
#pragma unroll
  for (int i = 0; i < NREG; ++i) {
    turn(i, ssum);
    ssum += chunk_sum(buf[i], nM);
  }
  for (int i = 0; i < n_lds; ++i) ssum += chunk_sum(mine_lds[i * NT], nM);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ssum += __shfl_xor(ssum, o, 64);
  if ((threadIdx.x & 63) == 0) sm_red[w] = ssum;                 // the maxima were all read before the second barrier
  __syncthreads();
  if (threadIdx.x == 0) {
    float Sx = 0.f;
    for (int i = 0; i < 8; ++i) Sx += sm_red[i];
    const float l = M + logf(Sx);
    lse[row] = l;
    loss_rows[row] = keep ? (l - sm_bc[2]) : 0.f;
    sm_bc[1] = l;
  }
  __syncthreads();
  if (!keep) {                                                   // uniform over the block
#pragma unroll
    for (int i = 0; i < NREG; ++i) store(zero4, off0, i * STEP * 2);
    for (int i = 0; i < n_lds; ++i) store(zero4, (uint32_t)(c0 + (NREG + i) * STEP) * 2u, 0);
    return;
  }
  float nl = -sm_bc[1] * LOG2E;
#pragma unroll
  for (int i = 0; i < NREG; ++i) {
    turn(i, nl);
    buf[i] = chunk_grad(buf[i], nl, sel_i == i);                 // takes the chunk's place: the next turn waits for it
    store(buf[i], off0, i * STEP * 2);
  }
  for (int i = 0; i < n_lds; ++i)
    store(chunk_grad(mine_lds[i * NT], nl, sel_i == NREG + i), (uint32_t)(c0 + (NREG + i) * STEP) * 2u, 0);
}

// 0 = take the resident-row kernel whenever the row fits; 1 = always the two-read kernel (for A/B timing)
#ifndef TIDE_CE_TWO_READS
#define TIDE_CE_TWO_READS 0
#endif
// most LDS chunks per thread the resident-row kernel is used with (8 = 64 KiB: two blocks per CU; up to 18 fit one block)
#ifndef TIDE_CE_MAX_LDS_CHUNKS
#define TIDE_CE_MAX_LDS_CHUNKS 18
#endif

hipError_t launch_ce_train(int64_t rows, int V, void* z, int64_t ldz, const int32_t* tokens, const uint8_t* mask,
                           float* lse, float* loss_rows, const int* rows_dev, int64_t rows_off, int dtype,
                           hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (ldz % 8 != 0) return hipErrorInvalidValue;
  ProfScope ps("ce_train", 0, (double)rows * ldz * 2.0 * dtype_size(dtype), s);
  if (rows_dev) prof_dynamic(rows_dev, rows_off, rows);
  constexpr size_t pad = 48 * 1024;   // occupancy limiter, see the kernel's comment
  dim3 grid((unsigned)rows), blk(512);
  const int ro = (int)rows_off;
  // resident-row kernel: chunks wholly below V go to registers (a template count, at most 24), the rest to LDS
  const int64_t nch = (ldz + 4095) / 4096, full = V / 4096;    // 16-byte chunks per thread of a 512-thread block
  static const int kRegs[] = {24, 20, 16, 12, 8, 4, 2, 1, 0};
  int nreg = 0;
  for (int r : kRegs)
    if (r <= full) { nreg = r; break; }
  const int64_t n_lds = nch - nreg;
  if (dtype == kBF16 && !TIDE_CE_TWO_READS && n_lds <= TIDE_CE_MAX_LDS_CHUNKS) {
    bf16_t* zb = (bf16_t*)z;
    dim3 blk_r(512);
    const size_t lds = (size_t)n_lds * 512 * 16;
    if (lds > 65536) {                          // only with 24 register chunks; one block per CU then
      static bool raised = false;
      if (!raised) {
        const hipError_t e = hipFuncSetAttribute((const void*)ce_train_resident_kernel<24>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 TIDE_CE_MAX_LDS_CHUNKS * 512 * 16);
        if (e != hipSuccess) return e;
        raised = true;
      }
    }
#define TIDE_CE_RES(R) case R: hipLaunchKernelGGL((ce_train_resident_kernel<R>), grid, blk_r, lds, s, zb, ldz, V, (int)n_lds, tokens, mask, lse, loss_rows, rows_dev, ro); break
    switch (nreg) {
      TIDE_CE_RES(24); TIDE_CE_RES(20); TIDE_CE_RES(16); TIDE_CE_RES(12); TIDE_CE_RES(8);
      TIDE_CE_RES(4); TIDE_CE_RES(2); TIDE_CE_RES(1); TIDE_CE_RES(0);
    }
#undef TIDE_CE_RES
    return hipGetLastError();
  }
  if (dtype == kBF16) hipLaunchKernelGGL(ce_train_kernel<bf16_t>, grid, blk, pad, s, (bf16_t*)z, ldz, V, tokens, mask, lse, loss_rows, rows_dev, ro);
  else hipLaunchKernelGGL(ce_train_kernel<float>, grid, blk, pad, s, (float*)z, ldz, V, tokens, mask, lse, loss_rows, rows_dev, ro);
  return hipGetLastError();
}

// loss = (1/N) * sum of loss_rows[0 .. *cnt) and, optionally, accuracy = (1/N) * sum of hit_rows[0 .. *cnt)
// (single block, fixed summation order: deterministic)
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ loss_rows,
                                                           const float* __restrict__ hit_rows,
                                                           const int* __restrict__ cnt,
                                                           const float* __restrict__ scal,
                                                           float* __restrict__ loss_out,
                                                           float* __restrict__ acc_out, int* __restrict__ status) {
  __shared__ float red[32];
  const int n = *cnt;
  float a = 0.f, h = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) {
    a += loss_rows[i];
    if (hit_rows) h += hit_rows[i];
  }
  const float tot = block_sum(a, red);
  if (threadIdx.x == 0) {
    const float loss = tot * scal[1];
    *loss_out = loss;
    if (!(fabsf(loss) <= 3.0e38f)) *status |= kStatusLossNotFinite;   // NaN or infinity (single thread: no race)
  }
  if (hit_rows && acc_out) {
    const float hits = block_sum(h, red);
    if (threadIdx.x == 0) *acc_out = hits * scal[1];
  }
}

hipError_t launch_loss_reduce(const float* loss_rows, const float* hit_rows, const int* cnt, const float* scal,
                              float* loss_out, float* acc_out, int* status, hipStream_t s) {
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, loss_rows, hit_rows, cnt, scal, loss_out, acc_out, status);
  return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// Fused multi-tensor AdamW.  One launch covers all tensors: block b works on 2048 x kAdamGroups consecutive
// elements of the tensor its index falls in (a thread owns kAdamGroups groups of 8, 2048 elements apart).  m, v and (bf16 mode) the master weights are fp32; the
// bf16 parameters are re-rounded from the master copy.  The caller passes 1/(1-beta1^t) and
// 1/sqrt(1-beta2^t) computed in double on the host.
// ----------------------------------------------------------------------------------------------
struct AdamDev {
  AdamTensor t[kMaxAdamTensors];
  int64_t blk_start[kMaxAdamTensors + 1];
  int nt;
  float lr, beta1, beta2, eps, decay, inv_bc1, inv_sqrt_bc2;
  const float* dyn;   // optional device {lr, decay, inv_bc1, inv_sqrt_bc2}
};

// The step-dependent scalars of AdamW computed on the device from a device-resident learning rate and step
// count, so that a captured training step replays with the values of the replay, not of the capture.
__global__ void adam_schedule_kernel(const float* __restrict__ lr_dev, int64_t* __restrict__ step_dev, float beta1,
                                     float beta2, float wd, float* __restrict__ dyn) {
  const long long t = (long long)(*step_dev + 1);
  const float lr = *lr_dev;
  dyn[0] = lr;
  dyn[1] = __fsub_rn(1.0f, __fmul_rn(lr, wd));   // two roundings, as the host computes it (no fused multiply-add)
  dyn[2] = (float)(1.0 / (1.0 - pow_int((double)beta1, t)));
  dyn[3] = (float)(1.0 / sqrt(1.0 - pow_int((double)beta2, t)));
  *step_dev += 1;
}

hipError_t launch_adam_schedule(const float* lr_dev, int64_t* step_dev, float beta1, float beta2, float wd, float* dyn,
                                hipStream_t s) {
  hipLaunchKernelGGL(adam_schedule_kernel, dim3(1), dim3(1), 0, s, lr_dev, step_dev, beta1, beta2, wd, dyn);
  return hipGetLastError();
}

#ifndef TIDE_ADAM_GROUPS
#define TIDE_ADAM_GROUPS 1
#endif
#ifndef TIDE_ADAM_NT_STORES
#define TIDE_ADAM_NT_STORES 0
#endif
constexpr int kAdamGroups = TIDE_ADAM_GROUPS;            // 8-element groups per thread, 256 * 8 elements apart
constexpr int kAdamPerBlock = 256 * 8 * kAdamGroups;     // elements per block

__device__ __forceinline__ void adam_store16(float4* p, const float4& v) {
#if TIDE_ADAM_NT_STORES
  typedef float f32x4_nt __attribute__((ext_vector_type(4)));
  f32x4_nt x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<f32x4_nt*>(p));
#else
  *p = v;
#endif
}

template <typename T>
__global__ __launch_bounds__(256) void adamw_kernel(AdamDev a) {
  int ti = 0;
  const int64_t b = blockIdx.x;
#pragma unroll
  for (int i = 1; i < kMaxAdamTensors; ++i)
    if (i < a.nt && b >= a.blk_start[i]) ti = i;
  const AdamTensor t = a.t[ti];
  const int64_t base = (b - a.blk_start[ti]) * kAdamPerBlock + threadIdx.x * 8;
  if (base >= t.n) return;
  T* p = (T*)t.p;
  float* w = (sizeof(T) == 2) ? t.master : (float*)t.p;
  const float omb1 = 1.f - a.beta1, omb2 = 1.f - a.beta2;
  // (locals: writing into the by-value argument would move the whole struct to scratch memory)
  const float lr = a.dyn ? a.dyn[0] : a.lr, decay = a.dyn ? a.dyn[1] : a.decay;
  const float inv_bc1 = a.dyn ? a.dyn[2] : a.inv_bc1, inv_sqrt_bc2 = a.dyn ? a.dyn[3] : a.inv_sqrt_bc2;
  if (base + (kAdamGroups - 1) * 2048 + 8 <= t.n) {
    // every load of the thread's groups is issued before the first value is used
    float g[kAdamGroups][8], m[kAdamGroups][8], v[kAdamGroups][8], th[kAdamGroups][8];
#pragma unroll
    for (int k = 0; k < kAdamGroups; ++k) {
      const int64_t i0 = base + k * 2048;
      ld8(t.g, i0, g[k]);
      ld8((const float*)t.m, i0, m[k]);
      ld8((const float*)t.v, i0, v[k]);
      ld8((const float*)w, i0, th[k]);
    }
#pragma unroll
    for (int k = 0; k < kAdamGroups; ++k) {
      const int64_t i0 = base + k * 2048;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        m[k][j] = a.beta1 * m[k][j] + omb1 * g[k][j];
        v[k][j] = a.beta2 * v[k][j] + omb2 * g[k][j] * g[k][j];
        const float denom = sqrtf(v[k][j]) * inv_sqrt_bc2 + a.eps;
        th[k][j] = th[k][j] * decay - lr * (m[k][j] * inv_bc1) / denom;
      }
      float4* qm = reinterpret_cast<float4*>(t.m + i0);
      float4* qv = reinterpret_cast<float4*>(t.v + i0);
      float4* qw = reinterpret_cast<float4*>(w + i0);
      adam_store16(qm, make_float4(m[k][0], m[k][1], m[k][2], m[k][3]));
      adam_store16(qm + 1, make_float4(m[k][4], m[k][5], m[k][6], m[k][7]));
      adam_store16(qv, make_float4(v[k][0], v[k][1], v[k][2], v[k][3]));
      adam_store16(qv + 1, make_float4(v[k][4], v[k][5], v[k][6], v[k][7]));
      adam_store16(qw, make_float4(th[k][0], th[k][1], th[k][2], th[k][3]));
      adam_store16(qw + 1, make_float4(th[k][4], th[k][5], th[k][6], th[k][7]));
      if (sizeof(T) == 2) st8(p, i0, th[k]);
    }
  } else {
    for (int k = 0; k < kAdamGroups; ++k)
      for (int64_t i = base + k * 2048; i < min(base + k * 2048 + 8, t.n); ++i) {
        const float g = t.g[i];
        const float m = a.beta1 * t.m[i] + omb1 * g;
        const float v = a.beta2 * t.v[i] + omb2 * g * g;
        const float denom = sqrtf(v) * inv_sqrt_bc2 + a.eps;
        const float th = w[i] * decay - lr * (m * inv_bc1) / denom;
        t.m[i] = m;
        t.v[i] = v;
        w[i] = th;
        if (sizeof(T) == 2) stf(p, i, th);
      }
  }
}

hipError_t launch_adamw(const AdamArgs& a, hipStream_t s) {
  AdamDev d;
  d.nt = a.nt;
  int64_t nb = 0;
  for (int i = 0; i < a.nt; ++i) {
    d.t[i] = a.t[i];
    d.blk_start[i] = nb;
    nb += (a.t[i].n + kAdamPerBlock - 1) / kAdamPerBlock;
  }
  for (int i = a.nt; i < kMaxAdamTensors; ++i) d.t[i] = AdamTensor{nullptr, nullptr, nullptr, nullptr, nullptr, 0};
  for (int i = a.nt; i <= kMaxAdamTensors; ++i) d.blk_start[i] = nb;
  d.lr = a.lr; d.beta1 = a.beta1; d.beta2 = a.beta2; d.eps = a.eps;
  d.decay = 1.0f - a.lr * a.wd;
  d.inv_bc1 = a.inv_bc1; d.inv_sqrt_bc2 = a.inv_sqrt_bc2;
  d.dyn = a.dyn;
  if (nb <= 0) return hipSuccess;
  double np_ = 0;
  for (int i = 0; i < a.nt; ++i) np_ += (double)a.t[i].n;
  ProfScope ps("adamw", 0, np_ * (a.dtype == kBF16 ? 30.0 : 28.0), s);
  if (a.dtype == kBF16) hipLaunchKernelGGL(adamw_kernel<bf16_t>, dim3((unsigned)nb), dim3(256), 0, s, d);
  else hipLaunchKernelGGL(adamw_kernel<float>, dim3((unsigned)nb), dim3(256), 0, s, d);
  return hipGetLastError();
}

}  // namespace tide

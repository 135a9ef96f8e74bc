// Device-side helpers shared by the gfx950 kernels of the TIDE draft-training step.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tide {

typedef uint16_t bf16_t;  // raw bfloat16 storage

constexpr int kWave = 64;  // CDNA wavefront width

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values in one instruction: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t f2bf2(float lo, float hi) {
  const hw_bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, size_t i) { return bf2f(p[i]); }
__device__ __forceinline__ void stf(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t* p, size_t i, float v) { p[i] = f2bf(v); }

// 8 consecutive elements <-> 8 floats (16-byte / 32-byte vector accesses; i must be a multiple of 8
// and the row base 16-byte aligned)
__device__ __forceinline__ void ld8(const float* p, size_t i, float (&v)[8]) {
  const float4* q = reinterpret_cast<const float4*>(p + i);
  float4 a = q[0], b = q[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void ld8(const bf16_t* p, size_t i, float (&v)[8]) {
  uint4 a = *reinterpret_cast<const uint4*>(p + i);
  uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[2 * j] = __uint_as_float(w[j] << 16);
    v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void st8(float* p, size_t i, const float (&v)[8]) {
  float4* q = reinterpret_cast<float4*>(p + i);
  q[0] = make_float4(v[0], v[1], v[2], v[3]);
  q[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void st8(bf16_t* p, size_t i, const float (&v)[8]) {
  uint32_t w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) w[j] = f2bf2(v[2 * j], v[2 * j + 1]);
  *reinterpret_cast<uint4*>(p + i) = make_uint4(w[0], w[1], w[2], w[3]);
}

// 8 consecutive elements as loaded, conversion to float deferred: a load whose value is not converted stays
// in flight until `get`, so it can overlap whatever is issued in between
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
  uint4 a;
  __device__ __forceinline__ void load(const bf16_t* p, size_t i) { a = *reinterpret_cast<const uint4*>(p + i); }
  __device__ __forceinline__ void zero() { a = make_uint4(0u, 0u, 0u, 0u); }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] = __uint_as_float(w[j] << 16);
      v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
    }
  }
};
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p, size_t i) {
    a = reinterpret_cast<const float4*>(p + i)[0];
    b = reinterpret_cast<const float4*>(p + i)[1];
  }
  __device__ __forceinline__ void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); b = a; }
  __device__ __forceinline__ void get(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block-wide sum for blocks of up to 1024 threads (a multiple of 64); every thread gets the result.
// `red` is LDS scratch of at least 17 floats.  Contains two barriers.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// The same sum with barriers that order LDS only.  __syncthreads() also waits for every global load the
// wave has in flight, which defeats a look-ahead; here loads issued before the call stay in flight across
// it.  Global stores of other threads are NOT made visible by this call.
__device__ __forceinline__ float block_sum_lds(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();            // everybody has read the previous result
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// The rows of sequence b: fixed-length batches keep sequence b in rows [b*Smax, (b+1)*Smax); packed batches
// give the row range through cu_seqlens (device, n_seqs+1 ascending offsets) and may hold empty sequences.
struct SeqView {
  int64_t row0;   // first row of the sequence in the [T, ...] activations
  int len;        // its length
};
// Packed: the offsets come from device memory the library cannot check on the host, so they are clamped
// here: whatever they hold, the view stays inside the T rows and is at most Smax long (no access can
// leave the buffers; a malformed list only gives wrong numbers, and the row plan raises a status bit).
__device__ __forceinline__ SeqView seq_view(const int* cu, int b, int Smax, int64_t T) {
  if (cu) {
    const int64_t s0 = min(max((int64_t)cu[b], (int64_t)0), T);
    const int64_t s1 = min(max((int64_t)cu[b + 1], s0), T);
    return SeqView{s0, (int)min(s1 - s0, (int64_t)Smax)};
  }
  return SeqView{(int64_t)b * Smax, Smax};
}
// index of (sequence b, head h, position i) in lse / delta: [B, nh, S] for fixed-length batches, [nh, T] packed
__device__ __forceinline__ size_t stat_index(const int* cu, int64_t T, const SeqView& v, int b, int h, int nh, int Smax, int i) {
  return cu ? (size_t)h * (size_t)T + (size_t)v.row0 + i : ((size_t)b * nh + h) * (size_t)Smax + i;
}

}  // namespace tide

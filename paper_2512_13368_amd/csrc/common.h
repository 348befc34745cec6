// Shared device-side helpers of the Blossom attention kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace blossom {

// Kernel-side problem description (passed by value).
struct KParams {
  int B, H, L, d;
  int b;        // block size
  int k;        // top-k (own block included)
  int w;        // short-term window
  int NB;       // ceil(L / b)
  float scale;  // softmax scale (already resolved, > 0)
  int sblk;     // mask block size of the full short-term mask (Eq. 15); 0 = local window only
  int last_lo;  // first of the last sblk positions (L - sblk); INT_MAX/2 when sblk == 0
  int nq;       // query blocks walked by select and forward: NB, or 1 (the last one) in serving mode
  int bidir;    // 1: bidirectional form (Eq. 15 as printed, no causal mask in either branch); sblk > 0 then
  // rotary position embedding (Sec. 3.3): cos/sin tables fp32 [L, d/2], or nullptr.  Backward kernels
  // then store dQ and dK rotated back (the gradient w.r.t. the rows before the rotation).
  const float *rope_cos, *rope_sin;
};

// ---- short-term mask, Eq. 15 in its causal form (callers guarantee j <= i, both valid) ----
__host__ __device__ __forceinline__ bool is_pow2(int x) { return x >= 1 && (x & (x - 1)) == 0; }
// does [lo, hi] hold a power of two (>= 1)?
__host__ __device__ __forceinline__ bool holds_pow2(int lo, int hi)
{
  if (hi < 1) return false;
  int top = 1;
  while (top <= hi / 2) top *= 2;  // largest power of two <= hi
  return top >= lo;
}
// (symmetric in i - j: the causal callers only ever ask about j <= i)
__device__ __forceinline__ bool st_visible(const KParams &p, int i, int j)
{
  if (abs(i - j) < p.w) return true;
  if (p.sblk == 0) return false;
  return j >= p.last_lo || is_pow2(abs(i / p.sblk - j / p.sblk));
}
// may any query of block I (size b) see any key of block J through the second or third case?
// (J <= I, or any J in the bidirectional form)
__device__ __forceinline__ bool st_block_reach(const KParams &p, int I, int J)
{
  if (p.sblk == 0) return false;
  const int q_lo = I * p.b, q_hi = min(I * p.b + p.b - 1, p.L - 1);
  const int k_lo = J * p.b, k_hi = min(J * p.b + p.b - 1, p.L - 1);
  if (k_hi >= p.last_lo) return true;
  if (J <= I) return holds_pow2(q_lo / p.sblk - k_hi / p.sblk, q_hi / p.sblk - k_lo / p.sblk);
  return holds_pow2(k_lo / p.sblk - q_hi / p.sblk, k_hi / p.sblk - q_lo / p.sblk);
}

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Round to nearest even; inputs are finite.
__device__ __forceinline__ uint16_t f32_to_bf16(float x)
{
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x.bits); }

template <typename T>
__device__ __forceinline__ T from_f32(float x);
template <>
__device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return bf16_t{f32_to_bf16(x)}; }

// Load 4 consecutive elements (16-byte aligned for fp32, 8-byte for bf16) as floats.
__device__ __forceinline__ void load4(const float *p, float (&o)[4])
{
  const float4 v = *reinterpret_cast<const float4 *>(p);
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void load4(const bf16_t *p, float (&o)[4])
{
  const uint2 v = *reinterpret_cast<const uint2 *>(p);
  o[0] = __uint_as_float(v.x << 16);
  o[1] = __uint_as_float(v.x & 0xFFFF0000u);
  o[2] = __uint_as_float(v.y << 16);
  o[3] = __uint_as_float(v.y & 0xFFFF0000u);
}
__device__ __forceinline__ void store4(float *p, const float (&o)[4])
{
  *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
}
__device__ __forceinline__ void store4(bf16_t *p, const float (&o)[4])
{
  uint2 v;
  v.x = (uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
  v.y = (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
  *reinterpret_cast<uint2 *>(p) = v;
}

__device__ __forceinline__ int clamp_len(int n, int L) { return n < 0 ? 0 : (n > L ? L : n); }

// Backward of the rotary position embedding on one channel pair (2i, 2i+1) of the row at position m:
// the transpose rotation, applied to the fp32 gradient before it is rounded to the storage type.
__device__ __forceinline__ void unrope_pair(const KParams &p, int m, int pair, int half_d, float &g0, float &g1)
{
  const float c = p.rope_cos[(size_t)m * half_d + pair], s = p.rope_sin[(size_t)m * half_d + pair];
  const float a = g0, b = g1;
  g0 = fmaf(c, a, s * b);
  g1 = fmaf(c, b, -(s * a));
}
template <int D>
__device__ __forceinline__ void unrope_row(const KParams &p, int m, float (&g)[D])
{
  if (!p.rope_cos) return;
#pragma unroll
  for (int i = 0; i < D / 2; ++i) unrope_pair(p, m, i, D / 2, g[2 * i], g[2 * i + 1]);
}

}  // namespace blossom

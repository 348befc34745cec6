// Ceilings of the matrix-core forward's tile loop, measured with that loop's own instruction mix
// and access patterns but without its bookkeeping (no masks, no reference moves, no tile list, no
// prologue or epilogue).  One launch runs `iters` tile steps per wavefront on every workgroup slot
// of the chip; the caller times the launch and divides.  The work of one step of one wavefront is
// the forward's steady-state tile for block size 64: 32 keys x 64 queries, d = 64, i.e. two
// matrix instructions that start the logits at minus the reference, eight for K Q^T, eight for
// V^T P^T, 32 exponentials with their bf16 conversions and row-sum adds, four 16-byte K fragment
// reads and eight transposing V fragment reads from LDS, and eight 1 KB global->LDS loads.
//   kind 0  matrix instructions only (operands in registers)
//   kind 1  softmax VALU work only
//   kind 2  both, operands in registers
//   kind 3  both, operands read from LDS tiles with the kernel's swizzled patterns
//   kind 4  all of it: plus double-buffered global->LDS staging of a K and a V tile per step
//   kind 5  the staging alone
// The K/V tiles are gathered pseudo-randomly from one head per XCD (2 MB, resident in that XCD's
// L2), which is the forward's own locality.
#include "../../include/blossom.h"

#include "launch.h"
#include "mfma_common.h"

namespace blossom {

using namespace mfma;

namespace {

constexpr int kProbeBlk = 64;
constexpr int kProbeTile = kProbeBlk * D;  // bf16 elements of a staged tile
constexpr int kProbeHalf = 32 * D;
constexpr int kProbeBlocks = 128;          // key blocks per head
constexpr int kProbeHeads = 8;             // one per XCD

constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

#define BLOSSOM_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

__device__ __forceinline__ float probe_expo(const f32x16 &s, bf16x8 (&pf)[2])
{
  float sa = 0.f, sb = 0.f;
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    const float pa = __builtin_amdgcn_exp2f(s[i]);
    const float pb = __builtin_amdgcn_exp2f(s[i + 1]);
    pf[i >> 3][i & 7] = (__bf16)pa;
    pf[i >> 3][(i & 7) + 1] = (__bf16)pb;
    sa += pa;
    sb += pb;
  }
  return sa + sb;
}

template <int KIND>
__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(2, 2))) void probe_kernel(
    const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, float *__restrict__ sink, int iters)
{
  __shared__ __attribute__((aligned(1024))) uint16_t Ks0[kProbeTile];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks1[kProbeTile];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs0[kProbeTile];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs1[kProbeTile];
  constexpr bool kMfma = KIND != 1 && KIND != 5, kValu = KIND != 0 && KIND != 5;
  constexpr bool kLds = KIND == 3 || KIND == 4, kStage = KIND == 4 || KIND == 5;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, lh = lane >> 5;
  const int bh = blockIdx.x % kProbeHeads;  // workgroup ids are dealt round-robin over the XCDs
  const size_t head = (size_t)bh * kProbeBlocks * kProbeTile;
  const char *Kh = reinterpret_cast<const char *>(K + head);
  const char *Vh = reinterpret_cast<const char *>(V + head);
  const int ld_row = 32 * wv + (lane >> 3);
  const unsigned k_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (lane >> 4)) * 8) * 2u;
  const unsigned v_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (2 * ((lane >> 3) & 3))) * 8) * 2u;
  auto stage = [&](const char *src_head, unsigned lane_off, unsigned odd_xor, uint16_t *dst_tile, int J)
                   __attribute__((always_inline)) {
    const char *src = src_head + (size_t)J * (kProbeTile * 2);
    lds_void *dst = (lds_void *)(dst_tile + 32 * wv * D);
    const unsigned lane_odd = lane_off ^ odd_xor;
    __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 1024, 0);
    __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 2048, 0);
    __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 3072, 0);
  };
  auto blk = [&](int t) -> int { return (int)(((unsigned)(t * 37 + blockIdx.x * 11)) % (unsigned)kProbeBlocks); };
  // both buffer pairs hold real tiles before the loop, whatever the kind
  stage(Kh, k_lane, 64u, Ks0, blk(0));
  stage(Vh, v_lane, 0u, Vs0, blk(0));
  stage(Kh, k_lane, 64u, Ks1, blk(1));
  stage(Vh, v_lane, 0u, Vs1, blk(1));
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

  bf16x8 qf[2][4], ones, mneg[2];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qf[0][kk][e] = (__bf16)(0.02f * (e - kk + lq));
      qf[1][kk][e] = (__bf16)(0.03f * (kk - e + lh));
    }
    ones[e] = (__bf16)((lh == 0 && e < 3) ? 1.f : 0.f);
    mneg[0][e] = (__bf16)(e < 3 ? -1.f : 0.f);
    mneg[1][e] = (__bf16)(e < 3 ? -2.f : 0.f);
  }
  int koff[4], voff[2];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = wv * kProbeHalf + lq * D + (((2 * kk + lh) ^ ((lq >> 1) & 7)) * 8);
  const int r16 = lane & 15;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
    voff[mb] = wv * kProbeHalf + (4 * lh + (r16 >> 2)) * D +
               (((4 * mb + 2 * ((lane >> 4) & 1) + ((r16 & 3) >> 1)) ^ (2 * (r16 >> 2))) * 8) + 4 * (r16 & 1);
  f32x16 oacc[2][2], zero16, sreg[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    zero16[i] = 0.f;
    sreg[0][i] = -0.01f * (float)(i + lq);
    sreg[1][i] = -0.02f * (float)(i + lh);
#pragma unroll
    for (int g = 0; g < 2; ++g) { oacc[g][0][i] = 0.f; oacc[g][1][i] = 0.f; }
  }
  float l_run[2] = {0.f, 0.f};
  int slow = 0;
  bf16x8 kreg[4], vreg[2][2], preg[2];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kreg[kk][e] = (__bf16)(0.01f * (e + kk + (lane & 7)));
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      preg[t][e] = (__bf16)(0.05f * (t + e));
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) vreg[t][mb][e] = (__bf16)(0.1f * (t + mb + e));
    }
  }
  auto tile = [&](const uint16_t *ks, const uint16_t *vs) __attribute__((always_inline)) {
    asm volatile("" : "+v"(koff[0]), "+v"(koff[1]), "+v"(koff[2]), "+v"(koff[3]), "+v"(voff[0]), "+v"(voff[1]));
    f32x16 s[2];
    if (kMfma) {
      s[0] = BLOSSOM_MFMA(ones, mneg[0], zero16);
      s[1] = BLOSSOM_MFMA(ones, mneg[1], zero16);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 kf;
        if (kLds) kf = *reinterpret_cast<const bf16x8 *>(ks + koff[kk]);
        else { kf = kreg[kk]; asm volatile("" : "+v"(kf)); }
        s[0] = BLOSSOM_MFMA(kf, qf[0][kk], s[0]);
        s[1] = BLOSSOM_MFMA(kf, qf[1][kk], s[1]);
      }
    } else {
      s[0] = sreg[0];
      s[1] = sreg[1];
      asm volatile("" : "+v"(s[0]), "+v"(s[1]));
    }
    bf16x8 vf[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        if (kLds) {
          const uint16_t *a0 = vs + 16 * t * D + voff[mb];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * D));
          vf[t][mb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
          vf[t][mb] = vreg[t][mb];
          asm volatile("" : "+v"(vf[t][mb]));
        }
      }
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      bf16x8 pf[2];
      if (kValu) {
        const float tsum = probe_expo(s[g], pf);
        if (__any(!(tsum <= 4096.f))) slow++;
        l_run[g] += tsum;
      } else {
        pf[0] = preg[0];
        pf[1] = preg[1];
        asm volatile("" : "+v"(pf[0]), "+v"(pf[1]));
        l_run[g] += s[g][0];
      }
      if (kMfma) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb) oacc[g][mb] = BLOSSOM_MFMA(vf[t][mb], pf[t], oacc[g][mb]);
      } else {
        l_run[g] += (float)pf[0][0] + (float)pf[1][7];
      }
    }
  };
  auto step = [&](int t, uint16_t *k_cur, uint16_t *v_cur, uint16_t *k_nxt, uint16_t *v_nxt) __attribute__((always_inline)) {
    if (kStage) {
      const int J = __builtin_amdgcn_readfirstlane(blk(t + 1));
      stage(Kh, k_lane, 64u, k_nxt, J);
      stage(Vh, v_lane, 0u, v_nxt, J);
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    }
    if (KIND != 5) tile(k_cur, v_cur);
  };
  for (int t = 0; t < iters; t += 2) {
    step(t, Ks0, Vs0, Ks1, Vs1);
    step(t + 1, Ks1, Vs1, Ks0, Vs0);
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  float r = l_run[0] + l_run[1] + (float)slow;
#pragma unroll
  for (int i = 0; i < 16; ++i) r += oacc[0][0][i] + oacc[0][1][i] + oacc[1][0][i] + oacc[1][1][i];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
}

}  // namespace
}  // namespace blossom

using namespace blossom;

extern "C" {

size_t blossom_probe_bytes(int which)
{
  if (which == 0) return (size_t)kProbeHeads * kProbeBlocks * kProbeTile * sizeof(uint16_t);  // K, and V
  if (which == 1) return (size_t)BLOSSOM_PROBE_WORKGROUPS * 128 * sizeof(float);               // sink
  return 0;
}

int blossom_probe(int kind, const void *K, const void *V, float *sink, int iters, void *hip_stream)
{
  if (!K || !V || !sink) return BLOSSOM_ERR_NULL;
  if (kind < 0 || kind > 5 || iters < 2 || iters > (1 << 20) || (iters & 1)) return BLOSSOM_ERR_PARAM;
  if ((reinterpret_cast<uintptr_t>(K) & 15u) || (reinterpret_cast<uintptr_t>(V) & 15u)) return BLOSSOM_ERR_ALIGN;
  (void)hipGetLastError();
  hipStream_t st = (hipStream_t)hip_stream;
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(BLOSSOM_PROBE_WORKGROUPS), dim3(128), 0, st, (const uint16_t *)K, (const uint16_t *)V,
                       sink, iters);
  };
  switch (kind) {
    case 0: go(probe_kernel<0>); break;
    case 1: go(probe_kernel<1>); break;
    case 2: go(probe_kernel<2>); break;
    case 3: go(probe_kernel<3>); break;
    case 4: go(probe_kernel<4>); break;
    default: go(probe_kernel<5>); break;
  }
  return hipGetLastError() == hipSuccess ? BLOSSOM_OK : BLOSSOM_ERR_LAUNCH;
}

}  // extern "C"

// The layer around the attention in one kernel (Sec. 2.1 Eq. 4: Concat(head_1..head_H) W^O; Sec. 3.6,
// the equation after Eq. 19: S = LayerNorm(H_prev + attention output), dropout being the identity):
//   z[b,t,n] = H_prev[b,t,n] + bias[n] + sum_{h,e} O[b,h,t,e] * Wt[n, h*d + e]
//   S[b,t,n] = (z - mean_n z) * rsqrt(var_n z + eps) * gamma[n] + beta[n]
// The attention output is read in the [B,H,L,d] layout the attention kernels write (the concatenation is
// only an address computation), the sum over all heads and channels stays in registers, and residual,
// bias, statistics and normalisation happen on the accumulators: no intermediate tensor touches HBM.
//
//  * outproj_mfma_kernel: bf16, d = 64, d_model 256 or 512, on v_mfma_f32_32x32x16_bf16.  Output
//    features are the M dimension and positions the N dimension, so a lane owns ONE position column and
//    the LayerNorm sums are in-lane adds plus one exchange with the lane that holds the column's other
//    features and one pass through LDS across the wavefronts.  Which weight row feeds which M row is
//    free: rows are dealt so that a lane ends up with 32 CONSECUTIVE features of its position, and
//    H_prev, bias, gamma, beta and S move as 16-byte pieces of a 64-byte run.
//  * outproj_generic_kernel: every other shape and fp32 storage, fp32 FMAs.
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

namespace {

// ------------------------------------------------------------------------------------------------
// scalar-ALU kernel: 256 threads = FT feature threads x PT position groups of 8 positions
// ------------------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;
constexpr int kGenPos = 8;  // positions per thread

__host__ __device__ inline int gen_feature_threads(int Dm) { return Dm <= 64 ? 64 : (Dm <= 128 ? 128 : 256); }
__host__ __device__ inline int gen_row_stride(int K, int Dm) { return (K > Dm ? K : Dm) + 4; }  // floats

template <typename T>
__global__ __launch_bounds__(kGenThreads) void outproj_generic_kernel(
    const T *__restrict__ O, const T *__restrict__ Wt, const float *__restrict__ bias, const T *__restrict__ Hprev,
    const float *__restrict__ gamma, const float *__restrict__ beta, float eps, T *__restrict__ S, float *__restrict__ mean_out,
    float *__restrict__ rstd_out, int B, int H, int L, int d, int Dm)
{
  extern __shared__ __attribute__((aligned(16))) float lds_op[];
  const int K = H * d;
  const int FT = gen_feature_threads(Dm);
  const int PT = kGenThreads / FT;
  const int TP = PT * kGenPos;  // positions of the workgroup
  const int LDR = gen_row_stride(K, Dm);
  const int tiles = (L + TP - 1) / TP;
  const int b = blockIdx.x / tiles, l0 = (blockIdx.x % tiles) * TP;
  const int tid = threadIdx.x;

  // the concatenated heads of TP positions as fp32 rows [pos][k]
  for (int i = tid; i < TP * (K / 4); i += kGenThreads) {
    const int e4 = i % (d / 4), rest = i / (d / 4);
    const int pos = rest % TP, h = rest / TP;
    const int t = min(l0 + pos, L - 1);
    float v[4];
    load4(O + (((size_t)b * H + h) * L + t) * d + 4 * e4, v);
    *reinterpret_cast<float4 *>(lds_op + pos * LDR + h * d + 4 * e4) = make_float4(v[0], v[1], v[2], v[3]);
  }
  __syncthreads();

  const int ft = tid % FT, pg = tid / FT;  // pg is uniform over a wavefront (FT >= 64)
  const float *crow = lds_op + pg * kGenPos * LDR;
  constexpr int NFMAX = 4;  // d_model <= 1024
  float acc[NFMAX][kGenPos];
#pragma unroll
  for (int j = 0; j < NFMAX; ++j)
#pragma unroll
    for (int q = 0; q < kGenPos; ++q) acc[j][q] = 0.0f;
#pragma unroll
  for (int j = 0; j < NFMAX; ++j) {
    const int n = ft + j * FT;
    if (n >= Dm) break;
    const T *wrow = Wt + (size_t)n * K;
    for (int k = 0; k < K; k += 4) {
      float w[4];
      load4(wrow + k, w);
#pragma unroll
      for (int q = 0; q < kGenPos; ++q) {
        const float4 c = *reinterpret_cast<const float4 *>(crow + q * LDR + k);
        acc[j][q] = fmaf(c.x, w[0], acc[j][q]);
        acc[j][q] = fmaf(c.y, w[1], acc[j][q]);
        acc[j][q] = fmaf(c.z, w[2], acc[j][q]);
        acc[j][q] = fmaf(c.w, w[3], acc[j][q]);
      }
    }
  }
  __syncthreads();  // every thread is done with the rows: they now take z

#pragma unroll
  for (int j = 0; j < NFMAX; ++j) {
    const int n = ft + j * FT;
    if (n >= Dm) break;
    const float bn = bias ? bias[n] : 0.0f;
#pragma unroll
    for (int q = 0; q < kGenPos; ++q) {
      const int pos = pg * kGenPos + q;
      const int t = min(l0 + pos, L - 1);
      lds_op[pos * LDR + n] = acc[j][q] + (to_f32(Hprev[((size_t)b * L + t) * Dm + n]) + bn);
    }
  }
  __syncthreads();

  // one wavefront per position at a time: two-pass statistics, then the normalised row
  const int lane = tid & 63, wv = tid >> 6;
  for (int pos = wv; pos < TP; pos += kGenThreads / 64) {
    const int t = l0 + pos;
    if (t >= L) break;  // (uniform over the wavefront)
    const float *z = lds_op + pos * LDR;
    float s = 0.0f;
    for (int n = lane; n < Dm; n += 64) s += z[n];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
    const float mean = s / (float)Dm;
    float v = 0.0f;
    for (int n = lane; n < Dm; n += 64) v = fmaf(z[n] - mean, z[n] - mean, v);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    const float rstd = 1.0f / sqrtf(v / (float)Dm + eps);
    T *out = S + ((size_t)b * L + t) * Dm;
    for (int n = lane; n < Dm; n += 64) out[n] = from_f32<T>(fmaf((z[n] - mean) * rstd, gamma[n], beta[n]));
    if (lane == 0) {
      if (mean_out) mean_out[(size_t)b * L + t] = mean;
      if (rstd_out) rstd_out[(size_t)b * L + t] = rstd;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// matrix-core kernel
// ------------------------------------------------------------------------------------------------
using namespace mfma;

constexpr int kOpWaves = 8;
constexpr int kOpPos = 128;            // positions of a workgroup
constexpr int kOpRowBytes = 144;       // a staged row: 64 bf16 + 16 bytes (rows of 36 words: 16-byte reads of 16 rows hit 64 distinct banks)
constexpr int kOpSlabBytes = kOpPos * kOpRowBytes;

// feature (relative to the wavefront's first) that row m of M block mb carries: lane half g = (m/4)%2 ends
// up holding, for its position, the 32 consecutive features 32 g + 16 mb + 4 (m/8) + m%4
__device__ __forceinline__ int op_feature(int mb, int m) { return 32 * ((m >> 2) & 1) + 16 * mb + 4 * (m >> 3) + (m & 3); }

template <int DM>
__global__ __launch_bounds__(64 * kOpWaves) void outproj_mfma_kernel(
    const uint16_t *__restrict__ O, const uint16_t *__restrict__ Wt, const float *__restrict__ bias,
    const uint16_t *__restrict__ Hprev, const float *__restrict__ gamma, const float *__restrict__ beta, float eps,
    uint16_t *__restrict__ S, float *__restrict__ mean_out, float *__restrict__ rstd_out, int B, int H, int L)
{
  constexpr int FW = DM / 64;          // feature groups (wavefronts side by side over the features)
  constexpr int PH = kOpWaves / FW;    // position parts (1 or 2)
  constexpr int NBW = (kOpPos / 32) / PH;  // 32-position N blocks per wavefront (4 or 2)
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  float *red1 = reinterpret_cast<float *>(lds_raw + 2 * kOpSlabBytes);  // [FW][128] sums
  float *red2 = red1 + FW * kOpPos;                                      // [FW][128] squared deviations

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wv % FW, wp = wv / FW;
  const int c = lane & 31, g = lane >> 5;
  const int K = H * 64;
  const int tiles = (L + kOpPos - 1) / kOpPos;
  const int b = blockIdx.x / tiles, l0 = (blockIdx.x % tiles) * kOpPos;
  const int fbase = wf * 64;
  const int pbase = wp * (NBW * 32);

  // staging: 1024 16-byte pieces per slab, two per thread (rows tid/8 and 64 + tid/8, piece tid%8)
  const int st_col = tid & 7;
  const uint16_t *st_src0 = O + ((size_t)b * H * L + min(l0 + (tid >> 3), L - 1)) * 64 + st_col * 8;  // head 0; a head
  const uint16_t *st_src1 = O + ((size_t)b * H * L + min(l0 + 64 + (tid >> 3), L - 1)) * 64 + st_col * 8;  // further is L*64 on
  const int st_dst0 = (tid >> 3) * kOpRowBytes + st_col * 16;
  const int st_dst1 = st_dst0 + 64 * kOpRowBytes;
  const size_t head_step = (size_t)L * 64;
  // this lane's weight rows (as supplier of row m = c of the two M blocks) at the k run 32 g .. 32 g + 31 of a slab
  const uint16_t *wsrc0 = Wt + (size_t)(fbase + op_feature(0, c)) * K + 32 * g;
  const uint16_t *wsrc1 = Wt + (size_t)(fbase + op_feature(1, c)) * K + 32 * g;

  f32x16 acc[2][NBW];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

  uint4 stage0, stage1;
  bf16x8 wcur[2][4], wnext[2][4];
  stage0 = *reinterpret_cast<const uint4 *>(st_src0);
  stage1 = *reinterpret_cast<const uint4 *>(st_src1);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    wcur[0][ks] = *reinterpret_cast<const bf16x8 *>(wsrc0 + 8 * ks);
    wcur[1][ks] = *reinterpret_cast<const bf16x8 *>(wsrc1 + 8 * ks);
  }
  *reinterpret_cast<uint4 *>(lds_raw + st_dst0) = stage0;
  *reinterpret_cast<uint4 *>(lds_raw + st_dst1) = stage1;
  __syncthreads();

  for (int h = 0; h < H; ++h) {
    const bool more = h + 1 < H;
    if (more) {  // the next head's rows and weights travel while this head is multiplied
      stage0 = *reinterpret_cast<const uint4 *>(st_src0 + (size_t)(h + 1) * head_step);
      stage1 = *reinterpret_cast<const uint4 *>(st_src1 + (size_t)(h + 1) * head_step);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        wnext[0][ks] = *reinterpret_cast<const bf16x8 *>(wsrc0 + (size_t)(h + 1) * 64 + 8 * ks);
        wnext[1][ks] = *reinterpret_cast<const bf16x8 *>(wsrc1 + (size_t)(h + 1) * 64 + 8 * ks);
      }
    }
    const unsigned char *rows = lds_raw + (h & 1) * kOpSlabBytes + (pbase + c) * kOpRowBytes + 64 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 of[NBW];
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) of[nb] = *reinterpret_cast<const bf16x8 *>(rows + nb * 32 * kOpRowBytes + 16 * ks);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wcur[mb][ks], of[nb], acc[mb][nb], 0, 0, 0);
    }
    if (more) {
      unsigned char *nxt = lds_raw + ((h + 1) & 1) * kOpSlabBytes;
      *reinterpret_cast<uint4 *>(nxt + st_dst0) = stage0;
      *reinterpret_cast<uint4 *>(nxt + st_dst1) = stage1;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) wcur[mb][ks] = wnext[mb][ks];
    }
    __syncthreads();
  }

  // epilogue: accumulator index 16 mb + 4 i + r of the lane is feature f0 + 16 mb + 4 i + r of position pbase + 32 nb + c
  const int f0 = fbase + 32 * g;
  float s1[NBW];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    const int t = min(l0 + pbase + 32 * nb + c, L - 1);
    const uint16_t *hp = Hprev + ((size_t)b * L + t) * DM + f0;
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {  // 8 features: M block q/2, rows i = 2 (q%2), 2 (q%2) + 1
      const uint4 hv = *reinterpret_cast<const uint4 *>(hp + 8 * q);
      const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w};
      float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (bias) {
        const float4 b0 = *reinterpret_cast<const float4 *>(bias + f0 + 8 * q);
        const float4 b1 = *reinterpret_cast<const float4 *>(bias + f0 + 8 * q + 4);
        bv[0] = b0.x; bv[1] = b0.y; bv[2] = b0.z; bv[3] = b0.w;
        bv[4] = b1.x; bv[5] = b1.y; bv[6] = b1.z; bv[7] = b1.w;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float hval = (e & 1) ? bf_hi(hw[e >> 1]) : bf_lo(hw[e >> 1]);
        const float a = acc[q >> 1][nb][8 * (q & 1) + e] + (hval + bv[e]);
        acc[q >> 1][nb][8 * (q & 1) + e] = a;
        s += a;
      }
    }
    s1[nb] = s + __shfl_xor(s, 32);  // with the lane that holds the other 32 features of the column
    if (g == 0) red1[wf * kOpPos + pbase + 32 * nb + c] = s1[nb];
  }
  __syncthreads();
  float mean[NBW], rstd[NBW];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    float s = 0.0f;
#pragma unroll
    for (int f = 0; f < FW; ++f) s += red1[f * kOpPos + pbase + 32 * nb + c];
    mean[nb] = s * (1.0f / (float)DM);
    float v = 0.0f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float dlt = acc[mb][nb][i] - mean[nb];
        v = fmaf(dlt, dlt, v);
      }
    v += __shfl_xor(v, 32);
    if (g == 0) red2[wf * kOpPos + pbase + 32 * nb + c] = v;
  }
  __syncthreads();
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    float v = 0.0f;
#pragma unroll
    for (int f = 0; f < FW; ++f) v += red2[f * kOpPos + pbase + 32 * nb + c];
    rstd[nb] = 1.0f / sqrtf(v * (1.0f / (float)DM) + eps);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float4 g0 = *reinterpret_cast<const float4 *>(gamma + f0 + 8 * q);
    const float4 g1 = *reinterpret_cast<const float4 *>(gamma + f0 + 8 * q + 4);
    const float4 e0 = *reinterpret_cast<const float4 *>(beta + f0 + 8 * q);
    const float4 e1 = *reinterpret_cast<const float4 *>(beta + f0 + 8 * q + 4);
    const float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const float bt[8] = {e0.x, e0.y, e0.z, e0.w, e1.x, e1.y, e1.z, e1.w};
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
      const int t = l0 + pbase + 32 * nb + c;
      if (t >= L) continue;
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        y[e] = fmaf((acc[q >> 1][nb][8 * (q & 1) + e] - mean[nb]) * rstd[nb], gm[e], bt[e]);
      uint4 o;
      o.x = pack2_bf16(y[0], y[1]);
      o.y = pack2_bf16(y[2], y[3]);
      o.z = pack2_bf16(y[4], y[5]);
      o.w = pack2_bf16(y[6], y[7]);
      *reinterpret_cast<uint4 *>(S + ((size_t)b * L + t) * DM + f0 + 8 * q) = o;
    }
  }
  if (wf == 0 && g == 0) {
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
      const int t = l0 + pbase + 32 * nb + c;
      if (t < L) {
        if (mean_out) mean_out[(size_t)b * L + t] = mean[nb];
        if (rstd_out) rstd_out[(size_t)b * L + t] = rstd[nb];
      }
    }
  }
}

size_t op_mfma_lds_bytes(int Dm) { return 2 * (size_t)kOpSlabBytes + 2 * (size_t)(Dm / 64) * kOpPos * sizeof(float); }

size_t op_generic_lds_bytes(int K, int Dm)
{
  const int TP = (kGenThreads / gen_feature_threads(Dm)) * kGenPos;
  return (size_t)TP * gen_row_stride(K, Dm) * sizeof(float);
}

bool op_mfma_shape(const OutProjArgs &a) { return a.dtype == 1 && a.d == 64 && (a.Dm == 256 || a.Dm == 512); }

}  // namespace

bool out_proj_supported(const OutProjArgs &a)
{
  if (op_mfma_shape(a)) return true;
  const long K = (long)a.H * a.d;
  return a.Dm >= 8 && a.Dm <= 1024 && a.Dm % 8 == 0 && K <= 1024 && op_generic_lds_bytes((int)K, a.Dm) <= 64 * 1024;
}

void launch_out_proj(const OutProjArgs &a, hipStream_t st)
{
  if (op_mfma_shape(a)) {
    const unsigned grid = (unsigned)(a.B * ((a.L + kOpPos - 1) / kOpPos));
    const size_t lds = op_mfma_lds_bytes(a.Dm);
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kOpWaves), lds, st, (const uint16_t *)a.O, (const uint16_t *)a.Wt,
                         a.bias, (const uint16_t *)a.Hprev, a.gamma, a.beta, a.eps, (uint16_t *)a.S, a.mean, a.rstd, a.B, a.H,
                         a.L);
    };
    if (a.Dm == 256) go(outproj_mfma_kernel<256>);
    else go(outproj_mfma_kernel<512>);
    return;
  }
  const int K = a.H * a.d;
  const int TP = (kGenThreads / gen_feature_threads(a.Dm)) * kGenPos;
  const unsigned grid = (unsigned)(a.B * ((a.L + TP - 1) / TP));
  const size_t lds = op_generic_lds_bytes(K, a.Dm);
  auto go = [&](auto kernel, auto tag) {
    using T = decltype(tag);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kGenThreads), lds, st, (const T *)a.O, (const T *)a.Wt, a.bias,
                       (const T *)a.Hprev, a.gamma, a.beta, a.eps, (T *)a.S, a.mean, a.rstd, a.B, a.H, a.L, a.d, a.Dm);
  };
  if (a.dtype == 0) go(outproj_generic_kernel<float>, float{});
  else go(outproj_generic_kernel<bf16_t>, bf16_t{});
}

}  // namespace blossom

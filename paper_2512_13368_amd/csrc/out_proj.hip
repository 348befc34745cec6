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

constexpr int kOpRowBytes = 144;       // a staged row: 64 bf16 + 16 bytes (rows of 36 words: 16-byte reads of 16 rows hit 64 distinct banks)
// One wavefront per 64 features, each over all positions of the workgroup: d_model 512 takes 8 wavefronts and 128
// positions (four 32-position blocks per wavefront, 128 accumulator registers, one workgroup per CU); d_model 256
// takes 4 wavefronts and 64 positions (two blocks, three workgroups per CU, whose load, multiply and store phases overlap).
template <int DM> struct OpGeo {
  static constexpr int kWaves = DM / 64;
  static constexpr int kPos = DM == 512 ? 128 : 64;
  static constexpr int kSlabBytes = kPos * kOpRowBytes;
};

// feature (relative to the wavefront's first) that row m of M block mb carries: lane half g = (m/4)%2 ends
// up holding, for its position, the 32 consecutive features 32 g + 16 mb + 4 (m/8) + m%4
__device__ __forceinline__ int op_feature(int mb, int m) { return 32 * ((m >> 2) & 1) + 16 * mb + 4 * (m >> 3) + (m & 3); }

template <int DM>
__global__ __launch_bounds__(64 * OpGeo<DM>::kWaves) void outproj_mfma_kernel(
    const uint16_t *__restrict__ O, const uint16_t *__restrict__ Wt, const float *__restrict__ bias,
    const uint16_t *__restrict__ Hprev, const float *__restrict__ gamma, const float *__restrict__ beta, float eps,
    uint16_t *__restrict__ S, float *__restrict__ mean_out, float *__restrict__ rstd_out, int B, int H, int L)
{
  constexpr int FW = OpGeo<DM>::kWaves;  // wavefronts side by side over the features
  constexpr int kOpPos = OpGeo<DM>::kPos, kOpSlabBytes = OpGeo<DM>::kSlabBytes;
  constexpr int NBW = kOpPos / 32;       // 32-position N blocks per wavefront (4 or 2)
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  float *red1 = reinterpret_cast<float *>(lds_raw + 2 * kOpSlabBytes);  // [FW][kOpPos] sums
  float *red2 = red1 + FW * kOpPos;                                      // [FW][kOpPos] squared deviations

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wv;
  const int c = lane & 31, g = lane >> 5;
  const int K = H * 64;
  const int tiles = (L + kOpPos - 1) / kOpPos;
  const int b = blockIdx.x / tiles, l0 = (blockIdx.x % tiles) * kOpPos;
  const int fbase = wf * 64;

  // staging: 8 16-byte pieces per row, two pieces per thread (rows tid/8 and kOpPos/2 + tid/8, piece tid%8)
  const int st_col = tid & 7;
  const uint16_t *st_src0 = O + ((size_t)b * H * L + min(l0 + (tid >> 3), L - 1)) * 64 + st_col * 8;  // head 0; a head
  const uint16_t *st_src1 = O + ((size_t)b * H * L + min(l0 + kOpPos / 2 + (tid >> 3), L - 1)) * 64 + st_col * 8;  // further is L*64 on
  const int st_dst0 = (tid >> 3) * kOpRowBytes + st_col * 16;
  const int st_dst1 = st_dst0 + (kOpPos / 2) * kOpRowBytes;
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
    const unsigned char *rows = lds_raw + (h & 1) * kOpSlabBytes + c * kOpRowBytes + 64 * g;
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

  // epilogue: accumulator index 16 mb + 4 i + r of the lane is feature f0 + 16 mb + 4 i + r of position 32 nb + c
  // H_prev comes in and S goes out through a 32-row area of LDS per wavefront (the slabs are free now): global
  // memory sees whole 128-byte rows (8 lanes each), the accumulator layout reads and writes its 16-byte pieces
  // there.  Only the wavefront itself touches its area: wave_barrier() orders its LDS writes and reads.
  const int f0 = fbase + 32 * g;
  unsigned char *area = lds_raw + wv * (32 * kOpRowBytes);
  const int er = lane >> 3, ec = lane & 7;  // as mover of whole rows: row 8 j + er, piece ec
  float s1[NBW];
  uint4 mv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t = min(l0 + 8 * j + er, L - 1);
    mv[j] = *reinterpret_cast<const uint4 *>(Hprev + ((size_t)b * L + t) * DM + fbase + 8 * ec);
  }
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(area + (8 * j + er) * kOpRowBytes + 16 * ec) = mv[j];
    if (nb + 1 < NBW) {  // the next block's rows travel meanwhile
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = min(l0 + 32 * (nb + 1) + 8 * j + er, L - 1);
        mv[j] = *reinterpret_cast<const uint4 *>(Hprev + ((size_t)b * L + t) * DM + fbase + 8 * ec);
      }
    }
    __builtin_amdgcn_wave_barrier();
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {  // 8 features: M block q/2, rows i = 2 (q%2), 2 (q%2) + 1
      const uint4 hv = *reinterpret_cast<const uint4 *>(area + c * kOpRowBytes + 64 * g + 16 * q);
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
    __builtin_amdgcn_wave_barrier();  // the area is read before the next block's rows land in it
    s1[nb] = s + __shfl_xor(s, 32);  // with the lane that holds the other 32 features of the column
    if (g == 0) red1[wf * kOpPos + 32 * nb + c] = s1[nb];
  }
  __syncthreads();
  float mean[NBW], rstd[NBW];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    float s = 0.0f;
#pragma unroll
    for (int f = 0; f < FW; ++f) s += red1[f * kOpPos + 32 * nb + c];
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
    if (g == 0) red2[wf * kOpPos + 32 * nb + c] = v;
  }
  __syncthreads();
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
    float v = 0.0f;
#pragma unroll
    for (int f = 0; f < FW; ++f) v += red2[f * kOpPos + 32 * nb + c];
    rstd[nb] = 1.0f / sqrtf(v * (1.0f / (float)DM) + eps);
  }
  float gm[4][8], bt[4][8];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float4 g0 = *reinterpret_cast<const float4 *>(gamma + f0 + 8 * q);
    const float4 g1 = *reinterpret_cast<const float4 *>(gamma + f0 + 8 * q + 4);
    const float4 e0 = *reinterpret_cast<const float4 *>(beta + f0 + 8 * q);
    const float4 e1 = *reinterpret_cast<const float4 *>(beta + f0 + 8 * q + 4);
    gm[q][0] = g0.x; gm[q][1] = g0.y; gm[q][2] = g0.z; gm[q][3] = g0.w;
    gm[q][4] = g1.x; gm[q][5] = g1.y; gm[q][6] = g1.z; gm[q][7] = g1.w;
    bt[q][0] = e0.x; bt[q][1] = e0.y; bt[q][2] = e0.z; bt[q][3] = e0.w;
    bt[q][4] = e1.x; bt[q][5] = e1.y; bt[q][6] = e1.z; bt[q][7] = e1.w;
  }
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        y[e] = fmaf((acc[q >> 1][nb][8 * (q & 1) + e] - mean[nb]) * rstd[nb], gm[q][e], bt[q][e]);
      uint4 o;
      o.x = pack2_bf16(y[0], y[1]);
      o.y = pack2_bf16(y[2], y[3]);
      o.z = pack2_bf16(y[4], y[5]);
      o.w = pack2_bf16(y[6], y[7]);
      *reinterpret_cast<uint4 *>(area + c * kOpRowBytes + 64 * g + 16 * q) = o;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int t = l0 + 32 * nb + 8 * j + er;
      const uint4 o = *reinterpret_cast<const uint4 *>(area + (8 * j + er) * kOpRowBytes + 16 * ec);
      if (t < L) *reinterpret_cast<uint4 *>(S + ((size_t)b * L + t) * DM + fbase + 8 * ec) = o;
    }
    __builtin_amdgcn_wave_barrier();
  }
  if (wf == 0 && g == 0) {
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
      const int t = l0 + 32 * nb + c;
      if (t < L) {
        if (mean_out) mean_out[(size_t)b * L + t] = mean[nb];
        if (rstd_out) rstd_out[(size_t)b * L + t] = rstd[nb];
      }
    }
  }
}

int op_mfma_pos(int Dm) { return Dm == 512 ? OpGeo<512>::kPos : OpGeo<256>::kPos; }
size_t op_mfma_lds_bytes(int Dm)
{
  return 2 * (size_t)op_mfma_pos(Dm) * kOpRowBytes + 2 * (size_t)(Dm / 64) * op_mfma_pos(Dm) * sizeof(float);
}

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
    const int tp = op_mfma_pos(a.Dm);
    const unsigned grid = (unsigned)(a.B * ((a.L + tp - 1) / tp));
    const size_t lds = op_mfma_lds_bytes(a.Dm);
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(a.Dm), lds, st, (const uint16_t *)a.O, (const uint16_t *)a.Wt,
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

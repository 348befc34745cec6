// Fused forward on the fp32 matrix instructions for short sequences (Eq. 1 under the two branch
// masks, Eq. 16-19, and the same-style dense causal comparison): fp32 storage, d = 32, block size 8 or
// 16, sequences whose K and V fit the LDS of a workgroup (L up to about 200: the paper's own regime,
// Sec. 4.1 / Appendix E: histories of at most 200 items, hidden size 64).
//
// One workgroup per (row, head).  K and V of the whole head are staged once into LDS (rows of 36
// floats: both operand read patterns below are bank-conflict free); each of the eight wavefronts then
// walks whole query blocks on its own, with no barrier and no staging inside the walks.  A query block
// is one 16-row tile of v_mfma_f32_16x16x4_f32 (block size 8 fills half of it), a key block one
// 16-key tile:
//   S^T = K Q^T   keys are the M dimension: lane (q = lane % 16, g = lane / 16) owns query column q and
//                 the logits of keys 4g .. 4g+3 of the tile; eight instructions (d = 32, 4 per step)
//   online softmax per column: in-lane over the 4 keys, two xor-shuffles over g
//   O^T += V^T P^T   P^T is the accumulator of S^T as it stands: step r contracts key 4g + r of every
//                 lane group, and V^T is read from LDS in exactly that key order; eight instructions
// The products are true fp32 products accumulated in fp32, so the fp32 tolerance of the scalar kernels
// holds.  Everything else (tile lists, masks, gate, outputs, padding rules) is what the scalar forward
// of generic.hip does; shapes outside this kernel's range stay there.
#include "launch.h"

namespace blossom {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D32 = 32;
constexpr int LDR = 36;            // floats per staged row
constexpr int kF32Waves = 8;
constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;
constexpr float kNegInfF = -__builtin_huge_valf();

// rows staged per tensor: every key block whole, plus the 16-key tile that starts at the last block
__host__ __device__ inline int f32_rows(const KParams &p) { return p.NB * p.b + 16; }

}  // namespace

template <int BK>
__global__ __launch_bounds__(64 * kF32Waves) void fwd_f32_mfma_kernel(
    const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V,
    const int *__restrict__ valid_len, const int *__restrict__ sel, const float *__restrict__ gate_w,
    const float *__restrict__ gate_b, float *__restrict__ O, float *__restrict__ o_lt_out,
    float *__restrict__ o_st_out, float *__restrict__ lse_lt_out, float *__restrict__ lse_st_out, int dense,
    KParams p)
{
  extern __shared__ __attribute__((aligned(16))) float lds_f32[];
  const int rows = f32_rows(p);
  float *Ks = lds_f32;
  float *Vs = lds_f32 + rows * LDR;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D32;

  // ---- K and V of the head into LDS (16-byte pieces, coalesced); rows past the end are zero ----
  for (int idx = tid; idx < rows * 8; idx += 64 * kF32Waves) {
    const int r = idx >> 3, c = idx & 7;
    float4 kx = make_float4(0.f, 0.f, 0.f, 0.f), vx = kx;
    if (r < p.L) {
      kx = *reinterpret_cast<const float4 *>(K + head + (size_t)r * D32 + 4 * c);
      vx = *reinterpret_cast<const float4 *>(V + head + (size_t)r * D32 + 4 * c);
    }
    *reinterpret_cast<float4 *>(Ks + r * LDR + 4 * c) = kx;
    *reinterpret_cast<float4 *>(Vs + r * LDR + 4 * c) = vx;
  }
  __syncthreads();

  const int q = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;
  const float bias = gate_b ? gate_b[h] : 0.0f;
  const int J_first = p0 / BK;

  // query blocks of this wavefront, longest walks first
  for (int idx = wv; idx < p.nq; idx += kF32Waves) {
    const int I = p.NB - 1 - idx;
    const int iq = I * BK + q;
    const bool in_range = q < BK && iq < p.L;
    const bool active = in_range && iq >= p0;
    const size_t rowoff = head + (size_t)min(iq, p.L - 1) * D32;
    const size_t lrow = (size_t)bh * p.L + min(iq, p.L - 1);

    if (min((I + 1) * BK, p.L) <= p0) {  // no valid query in the block: outputs are zero
      if (in_range) {
        const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          *reinterpret_cast<float4 *>(O + rowoff + 16 * mb + 4 * g) = z4;
          if (o_lt_out) *reinterpret_cast<float4 *>(o_lt_out + rowoff + 16 * mb + 4 * g) = z4;
          if (o_st_out) *reinterpret_cast<float4 *>(o_st_out + rowoff + 16 * mb + 4 * g) = z4;
        }
        if (g == 0) {
          if (lse_lt_out) lse_lt_out[lrow] = 0.0f;
          if (lse_st_out) lse_st_out[lrow] = 0.0f;
        }
      }
      continue;
    }

    // Q^T operand: lane (q, g) holds c*Q[iq][4s + g] for the eight steps s (zero for rows that take no part)
    float qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = active ? Q[rowoff + 4 * s + g] * c2 : 0.0f;
    // the selection row, 64 entries per register (requested now, used after the short-term branch)
    const int *my_sel = dense ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
    int sel_v = (!dense && lane < p.k) ? my_sel[lane] : -1;

    float m, l;
    f32x4 acc[2];
    auto reset = [&]() {
      m = kNegInfF;
      l = 0.0f;
      acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
      acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    // one tile: the 16 keys from position J*BK on (those of block J count) against the block's queries
    auto tile = [&](int J, bool windowed) {
      const float *kt = Ks + (J * BK + q) * LDR + g;   // row = key q of the tile (this lane's M index)
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < 8; ++st) s = __builtin_amdgcn_mfma_f32_16x16x4f32(kt[4 * st], qf[st], s, 0, 0, 0);
      // visible <=> key of block J, lo <= key <= iq (lo: start of the valid part, or of the window)
      const int lo = windowed ? max(p0, iq - p.w + 1) : p0;
      float mx = kNegInfF;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ko = 4 * g + r;
        const int key = J * BK + ko;
        const bool vis = active && ko < BK && key >= lo && key <= iq;
        s[r] = vis ? s[r] : kNegInfF;
        mx = fmaxf(mx, s[r]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx);
      const float m_use = m_new == kNegInfF ? 0.0f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m - m_use);  // 0 while nothing has been seen (acc and l are 0 then)
      float pr[4], psum = 0.0f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        pr[r] = __builtin_amdgcn_exp2f(s[r] - m_use);
        psum += pr[r];
      }
      l = l * alpha + psum;
      m = m_new;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mb][r] *= alpha;
      const float *vt = Vs + (J * BK + 4 * g) * LDR + q;  // row = key 4g + r, column = channel 16*mb + q
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(vt[r * LDR + 16 * mb], pr[r], acc[mb], 0, 0, 0);
    };
    // closes a branch: normalised output in acc (zero for rows that take no part), returns the lse
    auto finish = [&]() -> float {
      float lt = l + __shfl_xor(l, 16);
      lt += __shfl_xor(lt, 32);
      const bool ok = active && lt > 0.0f;
      const float inv = ok ? 1.0f / lt : 0.0f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mb][r] *= inv;
      return ok ? (m + __log2f(lt)) * kLn2F : 0.0f;
    };
    // acc[mb][r]: channel 16*mb + 4g + r of row iq
    auto store = [&](float *dst, const f32x4 (&a)[2]) {
      if (!in_range) return;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        *reinterpret_cast<float4 *>(dst + rowoff + 16 * mb + 4 * g) = make_float4(a[mb][0], a[mb][1], a[mb][2], a[mb][3]);
    };

    if (dense) {
      reset();
      for (int J = J_first; J <= I; ++J) tile(J, false);
      const float lse = finish();
      store(O, acc);
      if (in_range && g == 0 && lse_lt_out) lse_lt_out[lrow] = lse;
      continue;
    }

    // ---- short-term branch: causal window ----
    reset();
    {
      const int lowpos = I * BK - (p.w - 1);
      const int J_win = max(lowpos <= 0 ? 0 : lowpos / BK, J_first);
      for (int J = J_win; J <= I; ++J) tile(J, true);
    }
    const float lse_st = finish();
    const f32x4 ost[2] = {acc[0], acc[1]};

    // ---- long-term branch: selected blocks (entries outside [0, NB) are skipped) ----
    reset();
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      if (e0 > 0) sel_v = e0 + lane < p.k ? my_sel[e0 + lane] : -1;
      const int ne = min(64, p.k - e0);
      for (int e = 0; e < ne; ++e) {
        const int J = __builtin_amdgcn_readlane(sel_v, e);
        if (J < 0 || J >= p.NB) continue;
        tile(J, false);
      }
    }
    const float lse_lt = finish();

    // ---- gate and blend (Eq. 18-19) ----
    const float *wl = gate_w + (size_t)h * 2 * D32;
    float z = 0.0f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const float4 a = *reinterpret_cast<const float4 *>(wl + 16 * mb + 4 * g);
      const float4 b = *reinterpret_cast<const float4 *>(wl + D32 + 16 * mb + 4 * g);
      z = fmaf(a.x, acc[mb][0], z);
      z = fmaf(a.y, acc[mb][1], z);
      z = fmaf(a.z, acc[mb][2], z);
      z = fmaf(a.w, acc[mb][3], z);
      z = fmaf(b.x, ost[mb][0], z);
      z = fmaf(b.y, ost[mb][1], z);
      z = fmaf(b.z, ost[mb][2], z);
      z = fmaf(b.w, ost[mb][3], z);
    }
    z += __shfl_xor(z, 16);
    z += __shfl_xor(z, 32);
    z += bias;
    const float alpha = active ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
    if (o_lt_out) store(o_lt_out, acc);
    if (o_st_out) store(o_st_out, ost);
    f32x4 o[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) o[mb][r] = alpha * acc[mb][r] + (1.0f - alpha) * ost[mb][r];
    store(O, o);
    if (in_range && g == 0) {
      if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
      if (lse_st_out) lse_st_out[lrow] = lse_st;
    }
  }
}

bool fwd_f32_mfma_supported(const KParams &p, int dtype)
{
  return dtype == 0 && p.d == D32 && (p.b == 8 || p.b == 16) && p.sblk == 0 && !p.bidir &&
         2 * (size_t)f32_rows(p) * LDR * sizeof(float) <= 64 * 1024;
}

void launch_fwd_f32_mfma(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  const size_t lds = 2 * (size_t)f32_rows(p) * LDR * sizeof(float);
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3((unsigned)(p.B * p.H)), dim3(64 * kF32Waves), lds, st, (const float *)a.Q,
                       (const float *)a.K, (const float *)a.V, a.valid_len, a.sel, a.gate_w, a.gate_b, (float *)a.O,
                       (float *)a.o_lt, (float *)a.o_st, a.lse_lt, a.lse_st, a.dense, p);
  };
  if (p.b == 8) go(fwd_f32_mfma_kernel<8>);
  else go(fwd_f32_mfma_kernel<16>);
}

}  // namespace blossom

// Backward on the fp32 matrix instructions for short sequences: dQ (query-block stationary) and dK/dV
// (key-block stationary) for fp32 storage, d = 32, block size 8 or 16, with the streamed tensors of a
// whole head resident in LDS (the range of mfma_fwd_f32.hip; chain rule through Eq. 1 and Eq. 16-19 with
// the selection held fixed, as in the scalar kernels of generic.hip, whose per-row pass and inverse
// selection list feed these kernels too).
//
// With dO_x = a_x*dO + dz*Wg_x the upstream gradient of branch x (a_lt = alpha, a_st = 1 - alpha) and
// D_x = dO_x.o_x, both from the per-row pass:
//   P_ij = exp(scale*q_i.k_j - lse_x,i),  dS_ij = P_ij * (dO_x,i.v_j - D_x,i),
//   dQ_i = scale * sum_j dS_ij k_j,  dK_j = scale * sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_x,i.
// dO_x is never materialised: a lane forms the operand elements it feeds from dO, a_x, dz and Wg_x.
//
// One workgroup per (row, head), eight wavefronts, each walking whole blocks on its own, no barrier
// after the staging.  Tiles are 16 x 16 of v_mfma_f32_16x16x4_f32 (block size 8 fills half).
//   dQ:    keys are the M dimension (lane (q, g): query column q, keys 4g..4g+3), so lse and D_x are
//          per-lane scalars; S^T = K Q^T and G^T = V dO_x^T leave the matrix cores in the layout in
//          which dS^T is the B operand of dQ^T += K^T dS^T.  K, V in LDS.
//   dK/dV: queries are the M dimension (lane (key, g): key column, query rows 4g..4g+3); S = Q K^T,
//          G = dO_x V^T, then dV^T += dO_x^T P and dK^T += Q^T dS with P and dS as they stand.  Q, dO and
//          six per-row constants in LDS; the lane's own K and V rows in registers.
#include "launch.h"

namespace blossom {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D32 = 32;
constexpr int LDR = 36;  // floats per staged row: conflict-free for both operand read patterns
constexpr int kF32Waves = 8;
constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kHugeF = 1.0e30f;

__host__ __device__ inline int f32_rows(const KParams &p) { return p.NB * p.b + 16; }

// two tensors of a head into LDS, 16-byte pieces, rows past the end zero
__device__ __forceinline__ void stage_head(const float *__restrict__ A, const float *__restrict__ B, float *As,
                                           float *Bs, int rows, int L, int tid)
{
  for (int idx = tid; idx < rows * 8; idx += 64 * kF32Waves) {
    const int r = idx >> 3, c = idx & 7;
    float4 ax = make_float4(0.f, 0.f, 0.f, 0.f), bx = ax;
    if (r < L) {
      ax = *reinterpret_cast<const float4 *>(A + (size_t)r * D32 + 4 * c);
      bx = *reinterpret_cast<const float4 *>(B + (size_t)r * D32 + 4 * c);
    }
    *reinterpret_cast<float4 *>(As + r * LDR + 4 * c) = ax;
    *reinterpret_cast<float4 *>(Bs + r * LDR + 4 * c) = bx;
  }
}

// lane (col, g) holds channels 16*mb + 4g + r of row `pos` in a[mb][r]: scaled, rotated back when the
// caller's rows went through the rotary embedding (four consecutive channels = two channel pairs), stored
__device__ __forceinline__ void store_grad_row(float *dst, const f32x4 (&a)[2], float scale, const KParams &p, bool unrope,
                                               int pos, int g)
{
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    float v0 = a[mb][0] * scale, v1 = a[mb][1] * scale, v2 = a[mb][2] * scale, v3 = a[mb][3] * scale;
    if (unrope && p.rope_cos != nullptr) {
      const int pair = 8 * mb + 2 * g;
      unrope_pair(p, pos, pair, D32 / 2, v0, v1);
      unrope_pair(p, pos, pair + 1, D32 / 2, v2, v3);
    }
    *reinterpret_cast<float4 *>(dst + 16 * mb + 4 * g) = make_float4(v0, v1, v2, v3);
  }
}

}  // namespace

template <int BK>
__global__ __launch_bounds__(64 * kF32Waves) void bwd_dq_f32_mfma_kernel(
    const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V,
    const int *__restrict__ valid_len, const int *__restrict__ sel, const float *__restrict__ gate_w,
    const float *__restrict__ lse_lt, const float *__restrict__ lse_st, const float *__restrict__ dO,
    const float4 *__restrict__ rowstat, float *__restrict__ dQ, KParams p)
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
  stage_head(K + head, V + head, Ks, Vs, rows, p.L, tid);
  __syncthreads();

  const int q = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;
  const int J_first = p0 / BK;
  // this lane's slots of the two halves of the gate row: channel 4s + g for step s
  float wl[8], ws[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    wl[s] = gate_w[(size_t)h * 2 * D32 + 4 * s + g];
    ws[s] = gate_w[(size_t)h * 2 * D32 + D32 + 4 * s + g];
  }

  for (int idx = wv; idx < p.NB; idx += kF32Waves) {
    const int I = p.NB - 1 - idx;
    const int iq = I * BK + q;
    const bool in_range = q < BK && iq < p.L;
    const bool active = in_range && iq >= p0;
    const int row = min(iq, p.L - 1);
    const size_t rowoff = head + (size_t)row * D32;
    const size_t lrow = (size_t)bh * p.L + row;
    f32x4 dq[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    if (min((I + 1) * BK, p.L) <= p0) {  // no valid query in the block: zero gradients
      if (in_range) store_grad_row(dQ + rowoff, dq, 0.0f, p, false, row, g);
      continue;
    }
    float qf[8], gr[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      qf[s] = active ? Q[rowoff + 4 * s + g] * c2 : 0.0f;
      gr[s] = active ? dO[rowoff + 4 * s + g] : 0.0f;
    }
    const float4 st = active ? rowstat[lrow] : make_float4(0.f, 0.f, 0.f, 0.f);
    const float l2_lt = active ? lse_lt[lrow] * kLog2eF : kHugeF;  // rows that take no part: every probability zero
    const float l2_st = active ? lse_st[lrow] * kLog2eF : kHugeF;
    const int *my_sel = sel + ((size_t)bh * p.NB + I) * p.k;
    int sel_v = lane < p.k ? my_sel[lane] : -1;

    float gx[8];  // dO_x of the branch being walked
    float l2, Dx;
    auto tile = [&](int J, bool windowed) {
      const float *kt = Ks + (J * BK + q) * LDR + g;
      const float *vr = Vs + (J * BK + q) * LDR + g;
      f32x4 s = {0.f, 0.f, 0.f, 0.f}, gv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        s = __builtin_amdgcn_mfma_f32_16x16x4f32(kt[4 * t], qf[t], s, 0, 0, 0);
        gv = __builtin_amdgcn_mfma_f32_16x16x4f32(vr[4 * t], gx[t], gv, 0, 0, 0);
      }
      const int lo = windowed ? max(p0, iq - p.w + 1) : p0;
      float ds[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ko = 4 * g + r;
        const int key = J * BK + ko;
        const bool vis = active && ko < BK && key >= lo && key <= iq;
        ds[r] = vis ? __builtin_amdgcn_exp2f(s[r] - l2) * (gv[r] - Dx) : 0.0f;
      }
      const float *kc = Ks + (J * BK + 4 * g) * LDR + q;  // row = key 4g + r, column = channel 16*mb + q
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          dq[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kc[r * LDR + 16 * mb], ds[r], dq[mb], 0, 0, 0);
    };

    // short-term branch: causal window
#pragma unroll
    for (int s = 0; s < 8; ++s) gx[s] = fmaf(1.0f - st.x, gr[s], st.y * ws[s]);
    l2 = l2_st;
    Dx = st.w;
    {
      const int lowpos = I * BK - (p.w - 1);
      const int J_win = max(lowpos <= 0 ? 0 : lowpos / BK, J_first);
      for (int J = J_win; J <= I; ++J) tile(J, true);
    }
    // long-term branch: selected blocks
#pragma unroll
    for (int s = 0; s < 8; ++s) gx[s] = fmaf(st.x, gr[s], st.y * wl[s]);
    l2 = l2_lt;
    Dx = st.z;
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      if (e0 > 0) sel_v = e0 + lane < p.k ? my_sel[e0 + lane] : -1;
      const int ne = min(64, p.k - e0);
      for (int e = 0; e < ne; ++e) {
        const int J = __builtin_amdgcn_readlane(sel_v, e);
        if (J < 0 || J >= p.NB) continue;
        tile(J, false);
      }
    }
    if (in_range) store_grad_row(dQ + rowoff, dq, active ? p.scale : 0.0f, p, true, row, g);
  }
}

template <int BK>
__global__ __launch_bounds__(64 * kF32Waves) void bwd_dkv_f32_mfma_kernel(
    const float *__restrict__ Q, const float *__restrict__ K, const float *__restrict__ V,
    const int *__restrict__ valid_len, const float *__restrict__ gate_w, const float *__restrict__ lse_lt,
    const float *__restrict__ lse_st, const float *__restrict__ dO, const float4 *__restrict__ rowstat,
    const int *__restrict__ offs, const int *__restrict__ items, float *__restrict__ dK, float *__restrict__ dV,
    KParams p)
{
  extern __shared__ __attribute__((aligned(16))) float lds_f32[];
  const int rows = f32_rows(p);
  float *Qs = lds_f32;
  float *Gs = Qs + rows * LDR;      // dO rows
  float *rc = Gs + rows * LDR;      // per row: alpha, dz, D_lt, D_st, lse2_lt, lse2_st (six arrays of `rows`)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D32;
  stage_head(Q + head, dO + head, Qs, Gs, rows, p.L, tid);
  for (int r = tid; r < rows; r += 64 * kF32Waves) {
    float4 st = make_float4(0.f, 0.f, 0.f, 0.f);
    float a = kHugeF, b = kHugeF;  // rows that take no part: every probability zero
    if (r < p.L && r >= p0) {
      st = rowstat[(size_t)bh * p.L + r];
      a = lse_lt[(size_t)bh * p.L + r] * kLog2eF;
      b = lse_st[(size_t)bh * p.L + r] * kLog2eF;
    }
    rc[r] = st.x;
    rc[rows + r] = st.y;
    rc[2 * rows + r] = st.z;
    rc[3 * rows + r] = st.w;
    rc[4 * rows + r] = a;
    rc[5 * rows + r] = b;
  }
  __syncthreads();

  const int kq = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;
  // gate row: slot 4s + g for the products over channels, channel 16*mb + kq for the transposed operands
  float wl[8], ws[8], wlc[2], wsc[2];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    wl[s] = gate_w[(size_t)h * 2 * D32 + 4 * s + g];
    ws[s] = gate_w[(size_t)h * 2 * D32 + D32 + 4 * s + g];
  }
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    wlc[mb] = gate_w[(size_t)h * 2 * D32 + 16 * mb + kq];
    wsc[mb] = gate_w[(size_t)h * 2 * D32 + D32 + 16 * mb + kq];
  }
  const int *o = offs + (size_t)bh * (p.NB + 1);
  const int *it = items + (size_t)bh * p.NB * p.k;

  for (int J = wv; J < p.NB; J += kF32Waves) {  // early key blocks have the longest lists: they start first
    const int j = J * BK + kq;
    const bool in_range = kq < BK && j < p.L;
    const bool key_ok = in_range && j >= p0;
    const int row = min(j, p.L - 1);
    const size_t rowoff = head + (size_t)row * D32;
    f32x4 dk[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    f32x4 dv[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    if (min((J + 1) * BK, p.L) <= p0) {  // no valid key in the block
      if (in_range) {
        store_grad_row(dK + rowoff, dk, 0.0f, p, false, row, g);
        store_grad_row(dV + rowoff, dv, 0.0f, p, false, row, g);
      }
      continue;
    }
    float kf[8], vf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      kf[s] = key_ok ? K[rowoff + 4 * s + g] * c2 : 0.0f;
      vf[s] = key_ok ? V[rowoff + 4 * s + g] : 0.0f;
    }
    const int e_lo = o[J], e_hi = o[J + 1];

    // one tile: the 16 query rows from position I*BK on (those of block I count) against the block's keys
    auto tile = [&](int I, bool windowed) {
      const int r0 = I * BK;
      const float *ax_s = rc;                               // alpha
      const float *dz_s = rc + rows;
      const float *Dx_s = rc + (windowed ? 3 : 2) * rows;
      const float *l2_s = rc + (windowed ? 5 : 4) * rows;
      // S = Q K^T, G = dO_x V^T: this lane's A elements are those of query row r0 + kq
      const float *qt = Qs + (r0 + kq) * LDR + g;
      const float *gt = Gs + (r0 + kq) * LDR + g;
      const float al_m = ax_s[r0 + kq], dz_m = dz_s[r0 + kq];
      const float a_m = windowed ? 1.0f - al_m : al_m;
      f32x4 s = {0.f, 0.f, 0.f, 0.f}, gv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        s = __builtin_amdgcn_mfma_f32_16x16x4f32(qt[4 * t], kf[t], s, 0, 0, 0);
        gv = __builtin_amdgcn_mfma_f32_16x16x4f32(fmaf(a_m, gt[4 * t], dz_m * (windowed ? ws[t] : wl[t])), vf[t], gv, 0, 0, 0);
      }
      // visible <=> key valid, row of block I, key <= row, and (window) row - key < w; rows that take no
      // part carry an exponent of -1e30
      float pr[4], ds[4], a_r[4], dz_r[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int qo = 4 * g + r;
        const int i = r0 + qo;
        const bool vis = key_ok && qo < BK && i >= j && (!windowed || i - j < p.w);
        pr[r] = vis ? __builtin_amdgcn_exp2f(s[r] - l2_s[i]) : 0.0f;
        ds[r] = pr[r] * (gv[r] - Dx_s[i]);
        const float al = ax_s[i];
        a_r[r] = windowed ? 1.0f - al : al;
        dz_r[r] = dz_s[i];
      }
      // dV^T += dO_x^T P, dK^T += Q^T dS: row = query 4g + r, column = channel 16*mb + kq
      const float *gc = Gs + (r0 + 4 * g) * LDR + kq;
      const float *qc = Qs + (r0 + 4 * g) * LDR + kq;
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const float gxe = fmaf(a_r[r], gc[r * LDR + 16 * mb], dz_r[r] * (windowed ? wsc[mb] : wlc[mb]));
          dv[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(gxe, pr[r], dv[mb], 0, 0, 0);
          dk[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[r * LDR + 16 * mb], ds[r], dk[mb], 0, 0, 0);
        }
    };

    {  // short-term branch: query blocks whose window reaches this key block
      const long last_q = (long)J * BK + (BK - 1) + (p.w - 1);
      const int I_hi = (int)min((long)(p.NB - 1), last_q / BK);
      for (int I = J; I <= I_hi; ++I) tile(I, true);
    }
    // long-term branch: query blocks that selected this key block
    for (int e = e_lo; e < e_hi; ++e) {
      const int I = __builtin_amdgcn_readfirstlane(it[e]) & kInvBlockMask;
      tile(I, false);
    }
    if (in_range) {
      store_grad_row(dK + rowoff, dk, key_ok ? p.scale : 0.0f, p, true, row, g);
      store_grad_row(dV + rowoff, dv, key_ok ? 1.0f : 0.0f, p, false, row, g);
    }
  }
}

size_t bwd_f32_dkv_lds_bytes(const KParams &p) { return (size_t)f32_rows(p) * (2 * LDR + 6) * sizeof(float); }

bool bwd_f32_mfma_supported(const KParams &p, int dtype)
{
  return dtype == 0 && p.d == D32 && (p.b == 8 || p.b == 16) && p.sblk == 0 && !p.bidir &&
         2 * (size_t)f32_rows(p) * LDR * sizeof(float) <= 64 * 1024 && bwd_f32_dkv_lds_bytes(p) <= 96 * 1024;
}

void launch_bwd_f32_mfma(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st)
{
  const unsigned grid = (unsigned)(p.B * p.H);
  auto f = [](const void *x) { return reinterpret_cast<const float *>(x); };
  if (stages & kBwdStageDQ) {
    const size_t lds = 2 * (size_t)f32_rows(p) * LDR * sizeof(float);
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kF32Waves), lds, st, f(a.Q), f(a.K), f(a.V), a.valid_len, a.sel,
                         a.gate_w, a.lse_lt, a.lse_st, f(a.dO), w.rowstat, (float *)a.dQ, p);
    };
    if (p.b == 8) go(bwd_dq_f32_mfma_kernel<8>);
    else go(bwd_dq_f32_mfma_kernel<16>);
    if (launch_failed()) return;
  }
  if (stages & kBwdStageDKV) {
    const size_t lds = bwd_f32_dkv_lds_bytes(p);
    auto go = [&](auto kernel) {
      // (more than 64 KB of dynamic LDS has to be asked for; where it is not granted the launch fails and
      // the entry point reports it)
      if (lds > 64 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kF32Waves), lds, st, f(a.Q), f(a.K), f(a.V), a.valid_len, a.gate_w,
                         a.lse_lt, a.lse_st, f(a.dO), w.rowstat, w.offs, w.items, (float *)a.dK, (float *)a.dV, p);
    };
    if (p.b == 8) go(bwd_dkv_f32_mfma_kernel<8>);
    else go(bwd_dkv_f32_mfma_kernel<16>);
  }
}

}  // namespace blossom

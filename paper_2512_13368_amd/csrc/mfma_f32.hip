// Forward, dQ and dK/dV on the fp32 matrix instructions for short sequences (Eq. 1 under the two branch
// masks, Eq. 16-19 and their chain rule, and the same-style dense causal comparison): fp32 or bf16
// storage, d in {8, 16, 32}, block size 8 or 16, sequences whose streamed tensors fit the LDS of a
// workgroup.  That is the paper's own regime (Sec. 4.1, Appendix E: histories of at most 200 items,
// hidden size 64 over 2 to 8 heads, selection block 16); the 64 x 64 bf16 tiles of the long-sequence
// kernels would be mostly padding there.
//
// One workgroup per (row, head), eight wavefronts.  The tensors that a walk streams (K and V for
// forward and dQ, Q and dO for dK/dV) are staged once, as fp32, into LDS rows padded so that both
// operand read patterns below are bank-conflict free; each wavefront then walks whole blocks on its
// own, with no barrier and no staging inside the walks.  A block is one 16-row tile of
// v_mfma_f32_16x16x4_f32 (block size 8 fills half of it), products are true fp32 products accumulated
// in fp32, so the fp32 tolerance of the scalar kernels holds.
//   forward: S^T = K Q^T, keys as the M dimension: lane (q = lane % 16, g = lane / 16) owns query column
//            q and the logits of keys 4g .. 4g+3 of the tile; online softmax in-lane over the 4 keys plus
//            two xor-shuffles over g; O^T += V^T P^T with P^T = the accumulator of S^T as it stands (step
//            r contracts key 4g + r of every lane group, V^T is read from LDS in exactly that key order).
//   dQ:      same orientation, so lse and D_x are per-lane scalars; S^T and G^T = V dO_x^T leave the
//            matrix cores in the layout in which dS^T is the B operand of dQ^T += K^T dS^T.
//   dK/dV:   queries as the M dimension (lane (key, g): key column, query rows 4g .. 4g+3); S = Q K^T,
//            G = dO_x V^T, then dV^T += dO_x^T P and dK^T += Q^T dS with P and dS as they stand; six
//            per-row constants in LDS, the lane's own K and V rows in registers.
// With dO_x = a_x*dO + dz*Wg_x the upstream gradient of branch x (a_lt = alpha, a_st = 1 - alpha) and
// D_x = dO_x.o_x, both from the per-row pass of generic.hip:
//   P_ij = exp(scale*q_i.k_j - lse_x,i),  dS_ij = P_ij * (dO_x,i.v_j - D_x,i),
//   dQ_i = scale * sum_j dS_ij k_j,  dK_j = scale * sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_x,i;
// dO_x is never materialised: a lane forms the operand elements it feeds from dO, a_x, dz and Wg_x.
// Tile lists, masks (the causal window, or all of Eq. 15 in its causal or its bidirectional form), gate,
// outputs and padding rules are those of the scalar kernels of generic.hip; shapes outside this range stay there.
#include "launch.h"

namespace blossom {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kResWaves = 8;
constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;
constexpr float kNegInfF = -__builtin_huge_valf();
constexpr float kHugeF = 1.0e30f;
constexpr size_t kResLdsMax = 144 * 1024;

template <int D>
struct Geo {
  static constexpr int NS = D / 4;             // contraction steps over the channels (4 per instruction)
  static constexpr int NMB = (D + 15) / 16;    // 16-channel output blocks (d = 8 fills half of one)
  static constexpr int LDR = (D < 16 ? 16 : D) + 4;  // floats per staged row (20 or 36: conflict free, 16-byte rows)
};

// rows staged per tensor: every block whole, plus the 16-row tile that starts at the last block
__host__ __device__ inline int res_rows(const KParams &p) { return p.NB * p.b + 16; }

// two tensors of a head into LDS as fp32, 16-byte pieces; rows past the end and pad columns are zero
template <typename T, int D>
__device__ __forceinline__ void stage_head(const T *__restrict__ A, const T *__restrict__ B, float *As, float *Bs,
                                           int rows, int L, int tid)
{
  constexpr int CH = Geo<D>::LDR / 4;
  for (int idx = tid; idx < rows * CH; idx += 64 * kResWaves) {
    const int r = idx / CH, c = idx % CH;
    float ax[4] = {0.f, 0.f, 0.f, 0.f}, bx[4] = {0.f, 0.f, 0.f, 0.f};
    if (r < L && 4 * c < D) {
      load4(A + (size_t)r * D + 4 * c, ax);
      load4(B + (size_t)r * D + 4 * c, bx);
    }
    *reinterpret_cast<float4 *>(As + r * Geo<D>::LDR + 4 * c) = make_float4(ax[0], ax[1], ax[2], ax[3]);
    *reinterpret_cast<float4 *>(Bs + r * Geo<D>::LDR + 4 * c) = make_float4(bx[0], bx[1], bx[2], bx[3]);
  }
}

// lane (col, g) holds channels 16*mb + 4g + r of one row in a[mb][r]: stores those below D
template <typename T, int D>
__device__ __forceinline__ void store_row4(T *dst_row, const f32x4 (&a)[Geo<D>::NMB], int g)
{
#pragma unroll
  for (int mb = 0; mb < Geo<D>::NMB; ++mb)
    if (16 * mb + 4 * g < D) {
      const float v[4] = {a[mb][0], a[mb][1], a[mb][2], a[mb][3]};
      store4(dst_row + 16 * mb + 4 * g, v);
    }
}

// the same for a gradient row: scaled, rotated back when the caller's rows went through the rotary
// embedding (four consecutive channels = two channel pairs)
template <typename T, int D>
__device__ __forceinline__ void store_grad_row(T *dst_row, const f32x4 (&a)[Geo<D>::NMB], float scale, const KParams &p,
                                               bool unrope, int pos, int g)
{
#pragma unroll
  for (int mb = 0; mb < Geo<D>::NMB; ++mb)
    if (16 * mb + 4 * g < D) {
      float v[4] = {a[mb][0] * scale, a[mb][1] * scale, a[mb][2] * scale, a[mb][3] * scale};
      if (unrope && p.rope_cos != nullptr) {
        const int pair = 8 * mb + 2 * g;
        unrope_pair(p, pos, pair, D / 2, v[0], v[1]);
        unrope_pair(p, pos, pair + 1, D / 2, v[2], v[3]);
      }
      store4(dst_row + 16 * mb + 4 * g, v);
    }
}

// bidirectional form: last block the window of a row of block I reaches (key blocks of a query block, or
// query blocks of a key block: the window is symmetric)
__device__ __forceinline__ int window_reach_hi(int I, int b, int w, int NB)
{
  const long hi = (long)I * b + (b - 1) + (w - 1);
  return (int)min((long)(NB - 1), hi / b);
}

// element `c` of a gate-row half, zero past the head dimension
template <int D>
__device__ __forceinline__ float gate_at(const float *half, int c) { return c < D ? half[c] : 0.0f; }

}  // namespace

// =============================================================================================
// forward
// =============================================================================================
// PERPOS: the long-term branch takes one selection row per query POSITION and key/value group (the
// selection rule as printed, Eq. 8-13 with Eq. 4-5): K and V are [B,G,L,d], `sel` is [B,G,L,k] with
// selection blocks of BK positions; a lane folds its row into a bit per key block, and the walk visits the
// blocks any of the tile's rows selected, each row seeing its own.
template <typename T, int D, int BK, bool PERPOS>
__global__ __launch_bounds__(64 * kResWaves) void fwd_res_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, const int *__restrict__ valid_len,
    const int *__restrict__ sel, const float *__restrict__ gate_w, const float *__restrict__ gate_b,
    T *__restrict__ O, float *__restrict__ o_lt_out, float *__restrict__ o_st_out, float *__restrict__ lse_lt_out,
    float *__restrict__ lse_st_out, int dense, int kv_groups, KParams p)
{
  constexpr int NS = Geo<D>::NS, NMB = Geo<D>::NMB, LDR = Geo<D>::LDR;
  extern __shared__ __attribute__((aligned(16))) float lds_res[];
  const int rows = res_rows(p);
  float *Ks = lds_res;
  float *Vs = lds_res + rows * LDR;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D;
  // (grouped-query attention: head h reads the keys and values of group h / (H/G))
  const int kvh = PERPOS ? (bh / p.H) * kv_groups + h / (p.H / kv_groups) : bh;
  const size_t head_kv = (size_t)kvh * p.L * D;
  stage_head<T, D>(K + head_kv, V + head_kv, Ks, Vs, rows, p.L, tid);
  __syncthreads();

  const int q = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;
  const float bias = gate_b ? gate_b[h] : 0.0f;
  const int J_first = p0 / BK;

  // query blocks of this wavefront, longest walks first
  for (int idx = wv; idx < p.nq; idx += kResWaves) {
    const int I = p.NB - 1 - idx;
    const int iq = I * BK + q;
    const bool in_range = q < BK && iq < p.L;
    const bool active = in_range && iq >= p0;
    const size_t rowoff = head + (size_t)min(iq, p.L - 1) * D;
    const size_t lrow = (size_t)bh * p.L + min(iq, p.L - 1);

    f32x4 acc[NMB];
    if (min((I + 1) * BK, p.L) <= p0) {  // no valid query in the block: outputs are zero
      if (in_range) {
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb) acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        store_row4<T, D>(O + rowoff, acc, g);
        if (o_lt_out) store_row4<float, D>(o_lt_out + rowoff, acc, g);
        if (o_st_out) store_row4<float, D>(o_st_out + rowoff, acc, g);
        if (g == 0) {
          if (lse_lt_out) lse_lt_out[lrow] = 0.0f;
          if (lse_st_out) lse_st_out[lrow] = 0.0f;
        }
      }
      continue;
    }

    // Q^T operand: lane (q, g) holds c*Q[iq][4s + g] for the steps s (zero for rows that take no part)
    float qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = active ? to_f32(Q[rowoff + 4 * s + g]) * c2 : 0.0f;
    // the selection row, 64 entries per register (requested now, used after the short-term branch)
    const int *my_sel = (dense || PERPOS) ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
    int sel_v = (!dense && !PERPOS && lane < p.k) ? my_sel[lane] : -1;
    unsigned long long lt_mask = 0ull;  // PERPOS: bit J set iff this lane's position selected block J
    if (PERPOS && active) {
      const int *prow = sel + ((size_t)kvh * p.L + iq) * p.k;
      for (int e = 0; e < p.k; ++e) {
        const int v = prow[e];
        if (v >= 0 && v < p.NB) lt_mask |= 1ull << v;
      }
    }

    float m, l;
    auto reset = [&]() {
      m = kNegInfF;
      l = 0.0f;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb) acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    // one tile: the 16 keys from position J*BK on (those of block J count) against the block's queries
    auto tile = [&](int J, bool windowed) {
      const float *kt = Ks + (J * BK + q) * LDR + g;  // row = key q of the tile (this lane's M index)
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int st = 0; st < NS; ++st) s = __builtin_amdgcn_mfma_f32_16x16x4f32(kt[4 * st], qf[st], s, 0, 0, 0);
      float mx = kNegInfF;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ko = 4 * g + r;
        const int key = J * BK + ko;
        const bool vis = active && ko < BK && key >= p0 && key < p.L && (key <= iq || p.bidir) &&
                         (windowed ? st_visible(p, iq, key) : (!PERPOS || dense || ((lt_mask >> J) & 1ull)));
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
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mb][r] *= alpha;
      const float *vt = Vs + (J * BK + 4 * g) * LDR + q;  // row = key 4g + r, column = channel 16*mb + q
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb)
          acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(vt[r * LDR + 16 * mb], pr[r], acc[mb], 0, 0, 0);
    };
    // closes a branch: normalised output in acc (zero for rows that take no part), returns the lse
    auto finish = [&]() -> float {
      float lt = l + __shfl_xor(l, 16);
      lt += __shfl_xor(lt, 32);
      const bool ok = active && lt > 0.0f;
      const float inv = ok ? 1.0f / lt : 0.0f;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[mb][r] *= inv;
      return ok ? (m + __log2f(lt)) * kLn2F : 0.0f;
    };

    if (dense) {
      reset();
      for (int J = J_first; J <= I; ++J) tile(J, false);
      const float lse = finish();
      if (in_range) store_row4<T, D>(O + rowoff, acc, g);
      if (in_range && g == 0 && lse_lt_out) lse_lt_out[lrow] = lse;
      continue;
    }

    // ---- short-term branch: the causal window, and the blocks the other cases of Eq. 15 reach ----
    reset();
    {
      const int lowpos = I * BK - (p.w - 1);
      const int J_win = max(lowpos <= 0 ? 0 : lowpos / BK, J_first);
      for (int J = J_first; J < J_win; ++J)
        if (st_block_reach(p, I, J)) tile(J, true);
      for (int J = J_win; J <= I; ++J) tile(J, true);
      if (p.bidir) {  // Eq. 15 as printed: the same on the other side of the query block
        const int J_whi = window_reach_hi(I, BK, p.w, p.NB);
        for (int J = I + 1; J < p.NB; ++J)
          if (J <= J_whi || st_block_reach(p, I, J)) tile(J, true);
      }
    }
    const float lse_st = finish();
    f32x4 ost[NMB];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) ost[mb] = acc[mb];

    // ---- long-term branch: selected blocks (entries outside [0, NB) are skipped) ----
    reset();
    if (PERPOS) {
      for (int J = J_first; J <= I; ++J)
        if (__ballot((lt_mask >> J) & 1ull) != 0ull) tile(J, false);
    } else
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
    const float *wl = gate_w + (size_t)h * 2 * D;
    float z = 0.0f;
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = 16 * mb + 4 * g + r;
        z = fmaf(gate_at<D>(wl, c), acc[mb][r], z);
        z = fmaf(gate_at<D>(wl + D, c), ost[mb][r], z);
      }
    z += __shfl_xor(z, 16);
    z += __shfl_xor(z, 32);
    z += bias;
    const float alpha = active ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
    if (in_range) {
      if (o_lt_out) store_row4<float, D>(o_lt_out + rowoff, acc, g);
      if (o_st_out) store_row4<float, D>(o_st_out + rowoff, ost, g);
      f32x4 o[NMB];
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[mb][r] = alpha * acc[mb][r] + (1.0f - alpha) * ost[mb][r];
      store_row4<T, D>(O + rowoff, o, g);
      if (g == 0) {
        if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
        if (lse_st_out) lse_st_out[lrow] = lse_st;
      }
    }
  }
}

// =============================================================================================
// dQ
// =============================================================================================
// (PERPOS: as in the forward: `sel` is [B,G,L,k], K and V are [B,G,L,d])
template <typename T, int D, int BK, bool PERPOS>
__global__ __launch_bounds__(64 * kResWaves) void bwd_dq_res_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, const int *__restrict__ valid_len,
    const int *__restrict__ sel, const float *__restrict__ gate_w, const float *__restrict__ lse_lt,
    const float *__restrict__ lse_st, const T *__restrict__ dO, const float4 *__restrict__ rowstat, T *__restrict__ dQ,
    int kv_groups, KParams p)
{
  constexpr int NS = Geo<D>::NS, NMB = Geo<D>::NMB, LDR = Geo<D>::LDR;
  extern __shared__ __attribute__((aligned(16))) float lds_res[];
  const int rows = res_rows(p);
  float *Ks = lds_res;
  float *Vs = lds_res + rows * LDR;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D;
  const int kvh = PERPOS ? (bh / p.H) * kv_groups + h / (p.H / kv_groups) : bh;
  const size_t head_kv = (size_t)kvh * p.L * D;
  stage_head<T, D>(K + head_kv, V + head_kv, Ks, Vs, rows, p.L, tid);
  __syncthreads();

  const int q = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;
  const int J_first = p0 / BK;
  // this lane's slots of the two halves of the gate row: channel 4s + g for step s
  float wl[NS], ws[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    wl[s] = gate_w[(size_t)h * 2 * D + 4 * s + g];
    ws[s] = gate_w[(size_t)h * 2 * D + D + 4 * s + g];
  }

  for (int idx = wv; idx < p.NB; idx += kResWaves) {
    const int I = p.NB - 1 - idx;
    const int iq = I * BK + q;
    const bool in_range = q < BK && iq < p.L;
    const bool active = in_range && iq >= p0;
    const int row = min(iq, p.L - 1);
    const size_t rowoff = head + (size_t)row * D;
    const size_t lrow = (size_t)bh * p.L + row;
    f32x4 dq[NMB];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) dq[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (min((I + 1) * BK, p.L) <= p0) {  // no valid query in the block: zero gradients
      if (in_range) store_grad_row<T, D>(dQ + rowoff, dq, 0.0f, p, false, row, g);
      continue;
    }
    float qf[NS], gr[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      qf[s] = active ? to_f32(Q[rowoff + 4 * s + g]) * c2 : 0.0f;
      gr[s] = active ? to_f32(dO[rowoff + 4 * s + g]) : 0.0f;
    }
    const float4 st = active ? rowstat[lrow] : make_float4(0.f, 0.f, 0.f, 0.f);
    const float l2_lt = active ? lse_lt[lrow] * kLog2eF : kHugeF;  // rows that take no part: every probability zero
    const float l2_st = active ? lse_st[lrow] * kLog2eF : kHugeF;
    const int *my_sel = PERPOS ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
    int sel_v = (!PERPOS && lane < p.k) ? my_sel[lane] : -1;
    unsigned long long lt_mask = 0ull;  // PERPOS: bit J set iff this lane's position selected block J
    if (PERPOS && active) {
      const int *prow = sel + ((size_t)kvh * p.L + iq) * p.k;
      for (int e = 0; e < p.k; ++e) {
        const int v = prow[e];
        if (v >= 0 && v < p.NB) lt_mask |= 1ull << v;
      }
    }

    float gx[NS];  // dO_x of the branch being walked
    float l2, Dx;
    auto tile = [&](int J, bool windowed) {
      const float *kt = Ks + (J * BK + q) * LDR + g;
      const float *vr = Vs + (J * BK + q) * LDR + g;
      f32x4 s = {0.f, 0.f, 0.f, 0.f}, gv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < NS; ++t) {
        s = __builtin_amdgcn_mfma_f32_16x16x4f32(kt[4 * t], qf[t], s, 0, 0, 0);
        gv = __builtin_amdgcn_mfma_f32_16x16x4f32(vr[4 * t], gx[t], gv, 0, 0, 0);
      }
      float ds[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int ko = 4 * g + r;
        const int key = J * BK + ko;
        const bool vis = active && ko < BK && key >= p0 && key < p.L && (key <= iq || p.bidir) &&
                         (windowed ? st_visible(p, iq, key) : (!PERPOS || ((lt_mask >> J) & 1ull)));
        ds[r] = vis ? __builtin_amdgcn_exp2f(s[r] - l2) * (gv[r] - Dx) : 0.0f;
      }
      const float *kc = Ks + (J * BK + 4 * g) * LDR + q;  // row = key 4g + r, column = channel 16*mb + q
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb)
          dq[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kc[r * LDR + 16 * mb], ds[r], dq[mb], 0, 0, 0);
    };

    // short-term branch
#pragma unroll
    for (int s = 0; s < NS; ++s) gx[s] = fmaf(1.0f - st.x, gr[s], st.y * ws[s]);
    l2 = l2_st;
    Dx = st.w;
    {
      const int lowpos = I * BK - (p.w - 1);
      const int J_win = max(lowpos <= 0 ? 0 : lowpos / BK, J_first);
      for (int J = J_first; J < J_win; ++J)
        if (st_block_reach(p, I, J)) tile(J, true);
      for (int J = J_win; J <= I; ++J) tile(J, true);
      if (p.bidir) {  // Eq. 15 as printed: the same on the other side of the query block
        const int J_whi = window_reach_hi(I, BK, p.w, p.NB);
        for (int J = I + 1; J < p.NB; ++J)
          if (J <= J_whi || st_block_reach(p, I, J)) tile(J, true);
      }
    }
    // long-term branch: selected blocks
#pragma unroll
    for (int s = 0; s < NS; ++s) gx[s] = fmaf(st.x, gr[s], st.y * wl[s]);
    l2 = l2_lt;
    Dx = st.z;
    if (PERPOS) {
      for (int J = J_first; J <= I; ++J)
        if (__ballot((lt_mask >> J) & 1ull) != 0ull) tile(J, false);
    } else
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      if (e0 > 0) sel_v = e0 + lane < p.k ? my_sel[e0 + lane] : -1;
      const int ne = min(64, p.k - e0);
      for (int e = 0; e < ne; ++e) {
        const int J = __builtin_amdgcn_readlane(sel_v, e);
        if (J < 0 || J >= p.NB) continue;
        tile(J, false);
      }
    }
    if (in_range) store_grad_row<T, D>(dQ + rowoff, dq, active ? p.scale : 0.0f, p, true, row, g);
  }
}

// =============================================================================================
// dK, dV
// =============================================================================================
template <typename T, int D, int BK>
__global__ __launch_bounds__(64 * kResWaves) void bwd_dkv_res_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, const int *__restrict__ valid_len,
    const float *__restrict__ gate_w, const float *__restrict__ lse_lt, const float *__restrict__ lse_st,
    const T *__restrict__ dO, const float4 *__restrict__ rowstat, const int *__restrict__ offs,
    const int *__restrict__ items, T *__restrict__ dK, T *__restrict__ dV, KParams p)
{
  constexpr int NS = Geo<D>::NS, NMB = Geo<D>::NMB, LDR = Geo<D>::LDR;
  extern __shared__ __attribute__((aligned(16))) float lds_res[];
  const int rows = res_rows(p);
  float *Qs = lds_res;
  float *Gs = Qs + rows * LDR;  // dO rows
  float *rc = Gs + rows * LDR;  // per row: alpha, dz, D_lt, D_st, lse2_lt, lse2_st (six arrays of `rows`)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D;
  stage_head<T, D>(Q + head, dO + head, Qs, Gs, rows, p.L, tid);
  for (int r = tid; r < rows; r += 64 * kResWaves) {
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
  const float *wrow = gate_w + (size_t)h * 2 * D;
  float wl[NS], ws[NS], wlc[NMB], wsc[NMB];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    wl[s] = wrow[4 * s + g];
    ws[s] = wrow[D + 4 * s + g];
  }
#pragma unroll
  for (int mb = 0; mb < NMB; ++mb) {
    wlc[mb] = gate_at<D>(wrow, 16 * mb + kq);
    wsc[mb] = gate_at<D>(wrow + D, 16 * mb + kq);
  }
  const int *o = offs + (size_t)bh * (p.NB + 1);
  const int *it = items + (size_t)bh * p.NB * p.k;

  for (int J = wv; J < p.NB; J += kResWaves) {  // early key blocks have the longest lists: they start first
    const int j = J * BK + kq;
    const bool in_range = kq < BK && j < p.L;
    const bool key_ok = in_range && j >= p0;
    const int row = min(j, p.L - 1);
    const size_t rowoff = head + (size_t)row * D;
    f32x4 dk[NMB], dv[NMB];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) {
      dk[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (min((J + 1) * BK, p.L) <= p0) {  // no valid key in the block
      if (in_range) {
        store_grad_row<T, D>(dK + rowoff, dk, 0.0f, p, false, row, g);
        store_grad_row<T, D>(dV + rowoff, dv, 0.0f, p, false, row, g);
      }
      continue;
    }
    float kf[NS], vf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      kf[s] = key_ok ? to_f32(K[rowoff + 4 * s + g]) * c2 : 0.0f;
      vf[s] = key_ok ? to_f32(V[rowoff + 4 * s + g]) : 0.0f;
    }
    const int e_lo = o[J], e_hi = o[J + 1];

    // one tile: the 16 query rows from position I*BK on (those of block I count) against the block's keys
    auto tile = [&](int I, bool windowed) {
      const int r0 = I * BK;
      const float *ax_s = rc;  // alpha
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
      for (int t = 0; t < NS; ++t) {
        s = __builtin_amdgcn_mfma_f32_16x16x4f32(qt[4 * t], kf[t], s, 0, 0, 0);
        gv = __builtin_amdgcn_mfma_f32_16x16x4f32(fmaf(a_m, gt[4 * t], dz_m * (windowed ? ws[t] : wl[t])), vf[t], gv, 0, 0, 0);
      }
      // visible <=> key valid, row of block I, key <= row, and (short-term) the mask shows the pair; rows
      // that take no part carry an exponent of -1e30
      float pr[4], ds[4], a_r[4], dz_r[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int qo = 4 * g + r;
        const int i = r0 + qo;
        const bool vis = key_ok && qo < BK && (i >= j || p.bidir) && (!windowed || st_visible(p, i, j));
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
        for (int mb = 0; mb < NMB; ++mb) {
          const float gxe = fmaf(a_r[r], gc[r * LDR + 16 * mb], dz_r[r] * (windowed ? wsc[mb] : wlc[mb]));
          dv[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(gxe, pr[r], dv[mb], 0, 0, 0);
          dk[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[r * LDR + 16 * mb], ds[r], dk[mb], 0, 0, 0);
        }
    };

    {  // short-term branch: query blocks whose window reaches this key block, then those the other cases of Eq. 15 reach
      const long last_q = (long)J * BK + (BK - 1) + (p.w - 1);
      const int I_hi = (int)min((long)(p.NB - 1), last_q / BK);
      for (int I = J; I <= I_hi; ++I) tile(I, true);
      for (int I = I_hi + 1; I < p.NB; ++I)
        if (st_block_reach(p, I, J)) tile(I, true);
      if (p.bidir) {  // query blocks before the key block
        const int I_first = p0 / BK;
        const int lowpos = J * BK - (p.w - 1);
        const int I_lo = max(lowpos <= 0 ? 0 : lowpos / BK, I_first);
        for (int I = I_first; I < J; ++I)
          if (I >= I_lo || st_block_reach(p, I, J)) tile(I, true);
      }
    }
    // long-term branch: query blocks that selected this key block
    for (int e = e_lo; e < e_hi; ++e) {
      const int I = __builtin_amdgcn_readfirstlane(it[e]) & kInvBlockMask;
      tile(I, false);
    }
    if (in_range) {
      store_grad_row<T, D>(dK + rowoff, dk, key_ok ? p.scale : 0.0f, p, true, row, g);
      store_grad_row<T, D>(dV + rowoff, dv, key_ok ? 1.0f : 0.0f, p, false, row, g);
    }
  }
}

// =============================================================================================
// dK, dV under a per-position selection with grouped key/value heads: K, V, dK, dV are [B,G,L,d].
// One workgroup per (row, group).  The H/G query heads of the group all add into the same dK and dV,
// so a wavefront keeps the accumulators of its key block while the workgroup stages one head after
// the other (Q, dO and the per-row constants of that head), rounds of eight key blocks at a time.
// The selection rows of the group become one 64-bit word per position in LDS (bit J: block J
// selected) and their OR per query block: the long-term walk of key block J visits the query
// blocks whose word has bit J, each row testing its own.
// =============================================================================================
template <typename T, int D, int BK>
__global__ __launch_bounds__(64 * kResWaves) void bwd_dkv_pos_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, const int *__restrict__ valid_len,
    const int *__restrict__ sel_pos, const float *__restrict__ gate_w, const float *__restrict__ lse_lt,
    const float *__restrict__ lse_st, const T *__restrict__ dO, const float4 *__restrict__ rowstat, T *__restrict__ dK,
    T *__restrict__ dV, int kv_groups, KParams p)
{
  constexpr int NS = Geo<D>::NS, NMB = Geo<D>::NMB, LDR = Geo<D>::LDR;
  extern __shared__ __attribute__((aligned(16))) float lds_res[];
  const int rows = res_rows(p);
  float *Qs = lds_res;
  float *Gs = Qs + rows * LDR;  // dO rows
  float *rc = Gs + rows * LDR;  // per row: alpha, dz, D_lt, D_st, lse2_lt, lse2_st (six arrays of `rows`)
  unsigned long long *pmask = reinterpret_cast<unsigned long long *>(rc + 6 * rows);  // [rows] selection bits per position
  unsigned long long *bmask = pmask + rows;                                            // [NB] their OR per query block

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bg = blockIdx.x;               // (row, group)
  const int r_b = bg / kv_groups, grp = bg % kv_groups;
  const int hpg = p.H / kv_groups;         // query heads per group
  const int n = clamp_len(valid_len[r_b], p.L);
  const int p0 = p.L - n;
  const size_t head_kv = (size_t)bg * p.L * D;

  for (int i = tid; i < rows; i += 64 * kResWaves) {
    unsigned long long m = 0ull;
    if (i < p.L && i >= p0) {
      const int *prow = sel_pos + ((size_t)bg * p.L + i) * p.k;
      for (int e = 0; e < p.k; ++e) {
        const int v = prow[e];
        if (v >= 0 && v < p.NB) m |= 1ull << v;
      }
    }
    pmask[i] = m;
  }
  __syncthreads();
  for (int I = tid; I < p.NB; I += 64 * kResWaves) {
    unsigned long long m = 0ull;
    for (int t = 0; t < BK; ++t) m |= pmask[I * BK + t];
    bmask[I] = m;
  }

  const int kq = lane & 15, g = lane >> 4;
  const float c2 = p.scale * kLog2eF;

  for (int J0 = 0; J0 < p.NB; J0 += kResWaves) {  // rounds of eight key blocks, one per wavefront
    const int J = J0 + wv;
    const bool have = J < p.NB && min((J + 1) * BK, p.L) > p0;  // (uniform) a key block with a valid key
    const int j = J * BK + kq;
    const bool in_range = J < p.NB && kq < BK && j < p.L;
    const bool key_ok = in_range && j >= p0;
    const int row = min(max(j, 0), p.L - 1);
    const size_t rowoff = head_kv + (size_t)row * D;
    f32x4 dk[NMB], dv[NMB];
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) {
      dk[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float kf[NS], vf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      kf[s] = key_ok ? to_f32(K[rowoff + 4 * s + g]) * c2 : 0.0f;
      vf[s] = key_ok ? to_f32(V[rowoff + 4 * s + g]) : 0.0f;
    }

    for (int hh = 0; hh < hpg; ++hh) {
      const int h = grp * hpg + hh;
      const int bh = r_b * p.H + h;
      const size_t head = (size_t)bh * p.L * D;
      __syncthreads();  // every wavefront is done with the previous head's rows (and, the first time, bmask is written)
      stage_head<T, D>(Q + head, dO + head, Qs, Gs, rows, p.L, tid);
      for (int r = tid; r < rows; r += 64 * kResWaves) {
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
      if (!have) continue;

      const float *wrow = gate_w + (size_t)h * 2 * D;
      float wl[NS], ws[NS], wlc[NMB], wsc[NMB];
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        wl[s] = wrow[4 * s + g];
        ws[s] = wrow[D + 4 * s + g];
      }
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb) {
        wlc[mb] = gate_at<D>(wrow, 16 * mb + kq);
        wsc[mb] = gate_at<D>(wrow + D, 16 * mb + kq);
      }

      auto tile = [&](int I, bool windowed) {
        const int r0 = I * BK;
        const float *ax_s = rc;
        const float *dz_s = rc + rows;
        const float *Dx_s = rc + (windowed ? 3 : 2) * rows;
        const float *l2_s = rc + (windowed ? 5 : 4) * rows;
        const float *qt = Qs + (r0 + kq) * LDR + g;
        const float *gt = Gs + (r0 + kq) * LDR + g;
        const float al_m = ax_s[r0 + kq], dz_m = dz_s[r0 + kq];
        const float a_m = windowed ? 1.0f - al_m : al_m;
        f32x4 s = {0.f, 0.f, 0.f, 0.f}, gv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < NS; ++t) {
          s = __builtin_amdgcn_mfma_f32_16x16x4f32(qt[4 * t], kf[t], s, 0, 0, 0);
          gv = __builtin_amdgcn_mfma_f32_16x16x4f32(fmaf(a_m, gt[4 * t], dz_m * (windowed ? ws[t] : wl[t])), vf[t], gv, 0, 0, 0);
        }
        float pr[4], ds[4], a_r[4], dz_r[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int qo = 4 * g + r;
          const int i = r0 + qo;
          const bool vis = key_ok && qo < BK && i >= j &&
                           (windowed ? st_visible(p, i, j) : (((pmask[i] >> J) & 1ull) != 0ull));
          pr[r] = vis ? __builtin_amdgcn_exp2f(s[r] - l2_s[i]) : 0.0f;
          ds[r] = pr[r] * (gv[r] - Dx_s[i]);
          const float al = ax_s[i];
          a_r[r] = windowed ? 1.0f - al : al;
          dz_r[r] = dz_s[i];
        }
        const float *gc = Gs + (r0 + 4 * g) * LDR + kq;
        const float *qc = Qs + (r0 + 4 * g) * LDR + kq;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int mb = 0; mb < NMB; ++mb) {
            const float gxe = fmaf(a_r[r], gc[r * LDR + 16 * mb], dz_r[r] * (windowed ? wsc[mb] : wlc[mb]));
            dv[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(gxe, pr[r], dv[mb], 0, 0, 0);
            dk[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(qc[r * LDR + 16 * mb], ds[r], dk[mb], 0, 0, 0);
          }
      };

      {  // short-term branch of this head
        const long last_q = (long)J * BK + (BK - 1) + (p.w - 1);
        const int I_hi = (int)min((long)(p.NB - 1), last_q / BK);
        for (int I = J; I <= I_hi; ++I) tile(I, true);
        for (int I = I_hi + 1; I < p.NB; ++I)
          if (st_block_reach(p, I, J)) tile(I, true);
      }
      // long-term branch: query blocks with a position that selected this key block
      for (int I = J; I < p.NB; ++I)
        if ((bmask[I] >> J) & 1ull) tile(I, false);
    }
    if (in_range) {
      store_grad_row<T, D>(dK + rowoff, dk, key_ok ? p.scale : 0.0f, p, true, row, g);
      store_grad_row<T, D>(dV + rowoff, dv, key_ok ? 1.0f : 0.0f, p, false, row, g);
    }
  }
}

// =============================================================================================
// launchers
// =============================================================================================
namespace {

size_t res_kv_lds_bytes(const KParams &p, int D) { return 2 * (size_t)res_rows(p) * ((D < 16 ? 16 : D) + 4) * sizeof(float); }
size_t res_pos_dkv_lds_bytes(const KParams &p, int D)
{
  return res_kv_lds_bytes(p, D) + 6 * (size_t)res_rows(p) * sizeof(float) + ((size_t)res_rows(p) + p.NB) * sizeof(unsigned long long);
}
size_t res_dkv_lds_bytes(const KParams &p, int D) { return res_kv_lds_bytes(p, D) + 6 * (size_t)res_rows(p) * sizeof(float); }

bool res_shape(const KParams &p)
{
  // One workgroup per (row, head): enough of them to fill the chip, or so little work that it does not matter.
  // A mask block of Eq. 15 below the block size makes nearly every earlier block a short-term tile here (the
  // scalar kernels gather the few keys per row instead): only short sequences take that.
  return (p.d == 8 || p.d == 16 || p.d == 32) && (p.b == 8 || p.b == 16) &&
         ((long)p.B * p.H >= 64 || p.L <= 256) && (p.sblk == 0 || p.sblk >= p.b || p.L <= 256);
}

// (more than 64 KB of dynamic LDS has to be asked for; where it is not granted the launch fails and the
// entry point reports it)
template <typename Kern>
void want_lds(Kern kernel, size_t lds)
{
  if (lds > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

template <typename F>
void with_res_dims(const KParams &p, F &&f)
{
  auto with_bk = [&](auto dim) {
    if (p.b == 8) f(dim, std::integral_constant<int, 8>{});
    else f(dim, std::integral_constant<int, 16>{});
  };
  if (p.d == 8) with_bk(std::integral_constant<int, 8>{});
  else if (p.d == 16) with_bk(std::integral_constant<int, 16>{});
  else with_bk(std::integral_constant<int, 32>{});
}

}  // namespace

bool fwd_res_supported(const KParams &p, int dtype)
{
  (void)dtype;
  return res_shape(p) && res_kv_lds_bytes(p, p.d) <= kResLdsMax;
}

// the per-position form exists in this kernel family only: what the shape has to satisfy, whatever the batch
bool fwd_positions_supported(const KParams &p, int dtype)
{
  (void)dtype;
  return (p.d == 8 || p.d == 16 || p.d == 32) && (p.b == 8 || p.b == 16) && !p.bidir && p.NB <= 64 && p.nq == p.NB &&
         res_kv_lds_bytes(p, p.d) <= kResLdsMax;
}

bool bwd_res_supported(const KParams &p, int dtype)
{
  (void)dtype;
  // (d = 8 fills half of a 16-channel output block: measured, the scalar dK/dV pass is faster there)
  return res_shape(p) && p.d >= 16 && res_dkv_lds_bytes(p, p.d) <= kResLdsMax;
}

template <typename T>
static void launch_fwd_res_t(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  const size_t lds = res_kv_lds_bytes(p, p.d);
  with_res_dims(p, [&](auto dim, auto bk) {
    constexpr int D = decltype(dim)::value, BK = decltype(bk)::value;
    auto go = [&](auto kernel) {
      want_lds(kernel, lds);
      hipLaunchKernelGGL(kernel, dim3((unsigned)(p.B * p.H)), dim3(64 * kResWaves), lds, st, (const T *)a.Q, (const T *)a.K,
                         (const T *)a.V, a.valid_len, a.sel, a.gate_w, a.gate_b, (T *)a.O, (float *)a.o_lt, (float *)a.o_st,
                         a.lse_lt, a.lse_st, a.dense, a.kv_groups, p);
    };
    if (a.kv_groups > 0) go(fwd_res_kernel<T, D, BK, true>);
    else go(fwd_res_kernel<T, D, BK, false>);
  });
}

void launch_fwd_res(const KParams &p, int dtype, const FwdArgs &a, hipStream_t st)
{
  if (dtype == 0) launch_fwd_res_t<float>(p, a, st);
  else launch_fwd_res_t<bf16_t>(p, a, st);
}

template <typename T>
static void launch_bwd_res_t(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st)
{
  const unsigned grid = (unsigned)(p.B * p.H);
  with_res_dims(p, [&](auto dim, auto bk) {
    constexpr int D = decltype(dim)::value, BK = decltype(bk)::value;
    if (stages & kBwdStageDQ) {
      const size_t lds = res_kv_lds_bytes(p, p.d);
      auto kernel = bwd_dq_res_kernel<T, D, BK, false>;
      want_lds(kernel, lds);
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kResWaves), lds, st, (const T *)a.Q, (const T *)a.K, (const T *)a.V,
                         a.valid_len, a.sel, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO, w.rowstat, (T *)a.dQ, 0, p);
      if (launch_failed()) return;
    }
    if (stages & kBwdStageDKV) {
      const size_t lds = res_dkv_lds_bytes(p, p.d);
      auto kernel = bwd_dkv_res_kernel<T, D, BK>;
      want_lds(kernel, lds);
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * kResWaves), lds, st, (const T *)a.Q, (const T *)a.K, (const T *)a.V,
                         a.valid_len, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO, w.rowstat, w.offs, w.items, (T *)a.dK,
                         (T *)a.dV, p);
    }
  });
}

void launch_bwd_res(const KParams &p, int dtype, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st)
{
  if (dtype == 0) launch_bwd_res_t<float>(p, a, w, stages, st);
  else launch_bwd_res_t<bf16_t>(p, a, w, stages, st);
}

bool bwd_positions_supported(const KParams &p, int dtype)
{
  return fwd_positions_supported(p, dtype) && res_pos_dkv_lds_bytes(p, p.d) <= kResLdsMax;
}

// dQ [B,H,L,d] and dK, dV [B,G,L,d] under a per-position selection (a.sel = sel_pos [B,G,L,k]); the per-row pass
// has filled w.rowstat
template <typename T>
static void launch_bwd_pos_t(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, int kv_groups, hipStream_t st)
{
  with_res_dims(p, [&](auto dim, auto bk) {
    constexpr int D = decltype(dim)::value, BK = decltype(bk)::value;
    {
      const size_t lds = res_kv_lds_bytes(p, p.d);
      auto kernel = bwd_dq_res_kernel<T, D, BK, true>;
      want_lds(kernel, lds);
      hipLaunchKernelGGL(kernel, dim3((unsigned)(p.B * p.H)), dim3(64 * kResWaves), lds, st, (const T *)a.Q, (const T *)a.K,
                         (const T *)a.V, a.valid_len, a.sel, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO, w.rowstat,
                         (T *)a.dQ, kv_groups, p);
      if (launch_failed()) return;
    }
    {
      const size_t lds = res_pos_dkv_lds_bytes(p, p.d);
      auto kernel = bwd_dkv_pos_kernel<T, D, BK>;
      want_lds(kernel, lds);
      hipLaunchKernelGGL(kernel, dim3((unsigned)(p.B * kv_groups)), dim3(64 * kResWaves), lds, st, (const T *)a.Q,
                         (const T *)a.K, (const T *)a.V, a.valid_len, a.sel, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO,
                         w.rowstat, (T *)a.dK, (T *)a.dV, kv_groups, p);
    }
  });
}

void launch_bwd_positions(const KParams &p, int dtype, const BwdArgs &a, const BwdWorkspace &w, int kv_groups, hipStream_t st)
{
  if (dtype == 0) launch_bwd_pos_t<float>(p, a, w, kv_groups, st);
  else launch_bwd_pos_t<bf16_t>(p, a, w, kv_groups, st);
}

}  // namespace blossom

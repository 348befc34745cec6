// Backward on the matrix cores for bf16, d = 64, block size 32 or 64: dQ (query-block
// stationary) and dK/dV (key-block stationary), chain rule through Eq. 1 and Eq. 16-19 with
// the selection held fixed.
//
// The upstream gradient of branch x is dO_x = a_x*dO + dz*Wg_x (a_lt = alpha, a_st = 1-alpha;
// gate backward).  It is never materialised: rounding it to bf16 for the matrix cores would
// break the exact cancellation dS = P*(dO_x.v - dO_x.o) = 0 that rows with one key rely on.
// Everything the matrix cores see is an input tensor (Q, K, V, dO) or a probability; the gate
// enters through per-row and per-key scalars that the per-row pass leaves in the workspace:
//   dS_ij = P_ij * ( a_x[i]*(dO_i.v_j - dO_i.o_x,i) + dz[i]*(Wg_x.v_j - Wg_x.o_x,i) )
//   dV_j  = sum_i (a_x[i] P_ij) dO_i  +  Wg_x * sum_i dz[i] P_ij
// Accumulators start at minus a per-row constant, so the MFMA result is directly what the
// next step needs: the exponent S'' = c*q.k - lse*log2(e) (Q or K pre-multiplied by
// c = scale*log2(e)) and dO_i.v_j - dO_i.o_x,i.  Probabilities and dS leave the accumulator
// registers as the B operand of the next product without moving between lanes; the matching
// A operands (K^T, Q^T, dO^T) come from LDS through the transposing ds_read_b64_tr_b16.
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

using namespace mfma;

namespace {

// Per-lane LDS element offsets of the two operand read patterns for a tile staged with swz().
struct ReadOffsets {
  int row[4];  // row-per-lane 16-byte reads: slab kk; add 32*unit*D
  int tr[2];   // transposing 8-byte reads: M-block mb; add (32*unit + 16*t + 8*x)*D
};

__device__ __forceinline__ ReadOffsets read_offsets(int lane)
{
  ReadOffsets o;
  const int lq = lane & 31, lh = lane >> 5, r16 = lane & 15, g1 = (lane >> 4) & 1;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) o.row[kk] = lq * D + (((2 * kk + lh) ^ swz(lq)) * 8);
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
    o.tr[mb] = (4 * lh + (r16 >> 2)) * D +
               (((4 * mb + 2 * g1 + ((r16 & 3) >> 1)) ^ (2 * (r16 >> 2) + lh)) * 8) + 4 * (r16 & 1);
  return o;
}

// Direct global->LDS staging of one tile (BLK rows x 128 bytes): each wavefront moves 4 x 1 KB.
template <int BLK>
struct Stager {
  int wv, ld_row, over_base;
  bool ragged;
  int L, NB;
  __device__ __forceinline__ void init(int wv_, int lane, int L_, int NB_)
  {
    wv = wv_;
    L = L_;
    NB = NB_;
    ld_row = 32 * wv + (lane >> 3);
    ragged = L % BLK != 0;
  }
  // column (elements) of the chunk this lane fetches: LDS chunk position lane&7 holds chunk (lane&7)^swz(row)
  __device__ __forceinline__ static int lane_col(int lane) { return ((lane & 7) ^ (2 * ((lane >> 3) & 3) + ((lane >> 5) & 1))) * 8; }
  // src_lane = head + ld_row*D + lane_col
  __device__ __forceinline__ void stage(const uint16_t *src_lane, uint16_t *dst_tile, int blk) const
  {
    constexpr int TILE = BLK * D;
    if (!ragged || blk != NB - 1) {
      const uint16_t *src = src_lane + (size_t)blk * TILE;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        __builtin_amdgcn_global_load_lds((glb_void *)(src + 8 * u * D), (lds_void *)(dst_tile + (32 * wv + 8 * u) * D),
                                         16, 0, 0);
    } else {  // last, partial block: rows past the end are clamped (always masked)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int over = max(0, blk * BLK + ld_row + 8 * u - (L - 1));
        const uint16_t *src = src_lane + (size_t)blk * TILE + (8 * u - over) * D;
        __builtin_amdgcn_global_load_lds((glb_void *)src, (lds_void *)(dst_tile + (32 * wv + 8 * u) * D), 16, 0, 0);
      }
    }
  }
};

__device__ __forceinline__ bf16x8 lds_row(const uint16_t *tile, int off)
{
  return *reinterpret_cast<const bf16x8 *>(tile + off);
}

__device__ __forceinline__ bf16x8 lds_tr(const uint16_t *tile, int off)
{
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + off));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + off + 8 * D));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// 16 accumulator values -> two bf16 B operands (contraction halves t = 0, 1)
__device__ __forceinline__ void to_operand(const f32x16 &a, bf16x8 (&f)[2])
{
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    const bf16x2 pk = {(__bf16)a[i], (__bf16)a[i + 1]};
    f[i >> 3][i & 7] = pk[0];
    f[i >> 3][(i & 7) + 1] = pk[1];
  }
}

// row of bf16 (this lane's 4 slabs of 8) scaled by c, as the stationary operand
__device__ __forceinline__ void load_frags(const uint16_t *row, int lh, float c, bf16x8 (&f)[4])
{
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const uint4 raw = *reinterpret_cast<const uint4 *>(row + 16 * kk + 8 * lh);
    if (c == 1.0f) {
      f[kk] = __builtin_bit_cast(bf16x8, raw);
    } else {
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[kk][2 * e] = (__bf16)(bf_lo(w[e]) * c);
        f[kk][2 * e + 1] = (__bf16)(bf_hi(w[e]) * c);
      }
    }
  }
}

// store 2 x 16 accumulators (d x rows, transposed) of this lane's row as bf16, scaled
__device__ __forceinline__ void store_row_bf16(uint16_t *row, int lh, const f32x16 (&acc)[2], float scale, bool keep)
{
  if (!keep) {
#pragma unroll
    for (int c = 0; c < 32; c += 8) *reinterpret_cast<uint4 *>(row + 32 * lh + c) = make_uint4(0u, 0u, 0u, 0u);
    return;
  }
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = 32 * mb + 8 * g + 4 * lh;
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16(acc[mb][4 * g] * scale) | ((uint32_t)f32_to_bf16(acc[mb][4 * g + 1] * scale) << 16);
      pk.y = (uint32_t)f32_to_bf16(acc[mb][4 * g + 2] * scale) |
             ((uint32_t)f32_to_bf16(acc[mb][4 * g + 3] * scale) << 16);
      *reinterpret_cast<uint2 *>(row + d0) = pk;
    }
}

constexpr int kMaxTilesQ = 96;  // window blocks + selected blocks of one query block (host-checked)
constexpr int kFewKeys = 32;    // rows seeing fewer keys than this get two-term bf16 operands
constexpr float kBigProb = 0.03125f;  // a_x*P above this triggers the two-term operand in dK/dV

}  // namespace

// =============================================================================================
// dQ: one workgroup per (row, head, query block), one wavefront per 32 query rows.
//   per 32-key unit:  S''^T = K (cQ)^T - lse2     (keys x queries, lane owns a query column)
//                     G^T   = V dO^T - dO.o_x
//                     dS^T  = 2^S'' * (a_x*G^T + dz*(wv_x[key] - wo_x))  -> bf16 -> B operand
//                     dQ^T += K^T dS^T      (K^T through the transposing LDS read)
// =============================================================================================
template <int BLK>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_dq_mfma_kernel(const uint16_t *__restrict__ Q,
                                                              const uint16_t *__restrict__ K,
                                                              const uint16_t *__restrict__ V,
                                                              const int *__restrict__ valid_len,
                                                              const int *__restrict__ sel,
                                                              const float *__restrict__ lse_lt,
                                                              const float *__restrict__ lse_st,
                                                              const uint16_t *__restrict__ dO,
                                                              const float4 *__restrict__ rowstat,
                                                              const float4 *__restrict__ rowB,
                                                              const float2 *__restrict__ rowC,
                                                              uint16_t *__restrict__ dQ, KParams p)
{
  constexpr int UNITS = BLK / 32;
  constexpr int TILE = BLK * D;
  __shared__ __attribute__((aligned(1024))) uint16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs1[TILE];
  __shared__ __attribute__((aligned(16))) float wv_s[2][BLK];  // Wg_x.v_j of the staged key tiles
  __shared__ int tiles[kMaxTilesQ];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: MFMA regions must be scalar branches
  const int lq = lane & 31, lh = lane >> 5;
  const unsigned vid = xcd_remap(blockIdx.x, (unsigned)(p.B * p.H * p.NB));
  const int bh = (int)(vid / p.NB);
  const int I = p.NB - 1 - (int)(vid % p.NB);
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int q0 = I * BLK + 32 * wv;
  const int iq = q0 + lq;
  const bool q_ok = iq < p.L && iq >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t rowoff = head + (size_t)min(iq, p.L - 1) * D;
  const size_t lbase = (size_t)bh * p.L;
  const size_t lrow = lbase + min(iq, p.L - 1);

  f32x16 dq[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) { dq[0][i] = 0.0f; dq[1][i] = 0.0f; }
  if (min((I + 1) * BLK, p.L) <= p0) {  // no valid query: gradients are zero
    if (iq < p.L) store_row_bf16(dQ + rowoff, lh, dq, 0.0f, false);
    return;
  }

  const float c2 = p.scale * kLog2e;
  bf16x8 qf[4], gf[4];
  load_frags(Q + rowoff, lh, c2, qf);
  load_frags(dO + rowoff, lh, 1.0f, gf);
  // per-row constants; pad lanes get a huge lse so that every probability of their column is zero
  float lse2_lt = 1.0e30f, lse2_st = 1.0e30f;
  float a_lt = 0.0f, a_st = 0.0f, dz = 0.0f, do_lt = 0.0f, do_st = 0.0f, c0_lt = 0.0f, c0_st = 0.0f;
  if (q_ok) {
    const float4 st = rowstat[lrow];
    const float4 rb = rowB[lrow];
    lse2_lt = lse_lt[lrow] * kLog2e;
    lse2_st = lse_st[lrow] * kLog2e;
    a_lt = st.x;
    a_st = 1.0f - st.x;
    dz = st.y;
    do_lt = rb.x;
    do_st = rb.y;
    c0_lt = -dz * rb.z;
    c0_st = -dz * rb.w;
  }

  // ---- tile list: window blocks, then the selection list up to its first -1 ----
  const int J_first = p0 / BLK;
  const int lowpos = I * BLK - (p.w - 1);
  int J_lo = lowpos <= 0 ? 0 : lowpos / BLK;
  J_lo = max(J_lo, J_first);
  const int n_st = I - J_lo + 1;
  int n_lt = 0;
  bool lt_few = true;  // the selected past blocks hold fewer than kFewKeys valid keys
  {
    const int *my_sel = sel + ((size_t)bh * p.NB + I) * p.k;
    if (wv == 0)
      for (int t = lane; t < n_st; t += 64) tiles[t] = J_lo + t;
    bool open = true;
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      const int e = e0 + lane;
      const int J = e < p.k ? my_sel[e] : -1;
      const unsigned long long okm = __ballot(J >= 0 && J < p.NB);
      const int lead = okm == ~0ull ? 64 : __builtin_ctzll(~okm);
      if (open) {
        const bool mine = lane < lead;
        if (wv == 0 && mine) tiles[n_st + e] = J;
        const int vcount = min((J + 1) * BLK, p.L) - max(J * BLK, p0);
        if (__ballot(mine && J < I && vcount >= kFewKeys) != 0ull) lt_few = false;
        n_lt += lead;
        open = lead == 64;
      }
    }
  }
  // Rows with only a few keys: dq is a sum of a few large dS*k terms that nearly cancel, so the
  // bf16 rounding of dS would dominate it.  Such wavefronts feed dS as a two-term bf16 sum.
  const bool hp_st = p.w < kFewKeys || q0 - p0 + 1 < kFewKeys;
  const bool hp_lt = lt_few;
  const int n_all = n_st + n_lt;
  __syncthreads();
  auto tile_of = [&](int t) -> int { return __builtin_amdgcn_readfirstlane(tiles[t]); };

  Stager<BLK> sg;
  sg.init(wv, lane, p.L, p.NB);
  const uint16_t *k_lane = K + head + sg.ld_row * D + Stager<BLK>::lane_col(lane);
  const uint16_t *v_lane = V + head + sg.ld_row * D + Stager<BLK>::lane_col(lane);
  const ReadOffsets ro = read_offsets(lane);
  // Wg_x.v_j of key tile J for the branch the tile belongs to (0 past the end)
  auto key_const = [&](int J, bool windowed) __attribute__((always_inline)) -> float {
    float w = 0.0f;
    if (tid < BLK) {
      const int jj = J * BLK + tid;
      if (jj < p.L) {
        const float2 rc = rowC[lbase + jj];
        w = windowed ? rc.y : rc.x;
      }
    }
    return w;
  };

  auto tile_body = [&](const uint16_t *ks, const uint16_t *vs, const float *wvs, int J, bool windowed, float lse2,
                       float a_x, float do_x, float c0) __attribute__((always_inline)) {
    const bool hp = __builtin_amdgcn_readfirstlane((int)(windowed ? hp_st : hp_lt)) != 0;
    const bool masked = windowed || J == I || J * BLK < p0;
    const int lo = windowed ? max(p0, iq - p.w + 1) : p0;
    const unsigned span = (unsigned)(iq - lo);
    const bool any = iq >= lo;
#pragma unroll 1
    for (int s = 0; s < UNITS; ++s) {
      f32x16 sacc, gacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = -lse2; gacc[i] = -do_x; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(ks, 32 * s * D + ro.row[kk]), qf[kk], sacc, 0, 0, 0);
        gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(vs, 32 * s * D + ro.row[kk]), gf[kk], gacc, 0, 0, 0);
      }
      if (masked) {
        const int base = J * BLK + 32 * s + 4 * lh;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = base + 8 * (i >> 2) + (i & 3);
          const bool vis = any & ((unsigned)(key - lo) <= span);
          sacc[i] = vis ? sacc[i] : kNegInf;
        }
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 w4 = *reinterpret_cast<const float4 *>(wvs + 32 * s + 8 * g + 4 * lh);
        const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g + e;
          const float pr = __builtin_amdgcn_exp2f(sacc[i]);
          sacc[i] = pr * fmaf(a_x, gacc[i], fmaf(dz, w[e], c0));
        }
      }
      bf16x8 dsf[2];
      to_operand(sacc, dsf);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          dq[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(ks, (32 * s + 16 * t) * D + ro.tr[mb]), dsf[t],
                                                           dq[mb], 0, 0, 0);
      if (hp) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] -= (float)dsf[i >> 3][i & 7];
        to_operand(sacc, dsf);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
            dq[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(ks, (32 * s + 16 * t) * D + ro.tr[mb]), dsf[t],
                                                             dq[mb], 0, 0, 0);
      }
    }
  };

  {
    const int J0 = tile_of(0);
    sg.stage(k_lane, Ks0, J0);
    sg.stage(v_lane, Vs0, J0);
    const float w0 = key_const(J0, 0 < n_st);
    if (tid < BLK) wv_s[0][tid] = w0;
  }
  __syncthreads();
  auto step = [&](int t, uint16_t *k_fill, uint16_t *v_fill, const uint16_t *k_cur, const uint16_t *v_cur,
                  int par) __attribute__((always_inline)) {
    float wn = 0.0f;
    const bool more = t + 1 < n_all;
    if (more) {
      const int Jn = tile_of(t + 1);
      wn = key_const(Jn, t + 1 < n_st);
      sg.stage(k_lane, k_fill, Jn);
      sg.stage(v_lane, v_fill, Jn);
    }
    const bool win = t < n_st;
    tile_body(k_cur, v_cur, wv_s[par], tile_of(t), win, win ? lse2_st : lse2_lt, win ? a_st : a_lt,
              win ? do_st : do_lt, win ? c0_st : c0_lt);
    if (more && tid < BLK) wv_s[par ^ 1][tid] = wn;
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Ks1, Vs1, Ks0, Vs0, 0);
    if (t + 1 < n_all) step(t + 1, Ks0, Vs0, Ks1, Vs1, 1);
  }
  if (iq < p.L) store_row_bf16(dQ + rowoff, lh, dq, p.scale, q_ok);
}

// =============================================================================================
// dK, dV: one workgroup per (row, head, key block), one wavefront per 32 key rows; walks the
// query blocks whose window reaches the key block, then those that selected it (inverse list).
//   per 32-query unit:  S'' = Q (cK)^T - lse2[i]   (queries x keys, lane owns a key column)
//                       G   = dO V^T - dO.o_x[i]
//                       P = 2^S'',  dS = P*(a_x[i]*G + dz[i]*(wv_x[key] - wo_x[i]))
//                       dV^T += dO^T (a_x P),  u += dz[i]*P,  dK^T += Q^T dS
//   epilogue:           dV_j += Wg_lt*u_lt + Wg_st*u_st
// =============================================================================================
constexpr int kListRing = 128;

template <int BLK>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_dkv_mfma_kernel(const uint16_t *__restrict__ Q,
                                                               const uint16_t *__restrict__ K,
                                                               const uint16_t *__restrict__ V,
                                                               const int *__restrict__ valid_len,
                                                               const float *__restrict__ gate_w,
                                                               const float *__restrict__ lse_lt,
                                                               const float *__restrict__ lse_st,
                                                               const uint16_t *__restrict__ dO,
                                                               const float4 *__restrict__ rowstat,
                                                               const float4 *__restrict__ rowB,
                                                               const float2 *__restrict__ rowC,
                                                               const int *__restrict__ offs,
                                                               const int *__restrict__ items,
                                                               uint16_t *__restrict__ dK,
                                                               uint16_t *__restrict__ dV, KParams p)
{
  constexpr int UNITS = BLK / 32;
  constexpr int TILE = BLK * D;
  constexpr int NT = BLK * 2;
  __shared__ __attribute__((aligned(1024))) uint16_t Qs0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Qs1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Gs0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Gs1[TILE];
  // per-row constants of the staged query tile: lse2, dO.o_x, a_x, dz, -dz*wo_x
  __shared__ __attribute__((aligned(16))) float rc_s[2][5][BLK];
  __shared__ float gate_s[2 * D];
  __shared__ int ring[kListRing];  // query blocks of the long-term part of the walk, refilled in halves

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, lh = lane >> 5;
  const unsigned vid = xcd_remap(blockIdx.x, (unsigned)(p.B * p.H * p.NB));
  const int bh = (int)(vid / p.NB);
  const int h = bh % p.H;
  const int J = (int)(vid % p.NB);  // early key blocks are selected by more query blocks: start them first
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int j = J * BLK + 32 * wv + lq;  // this lane's key row
  const bool key_ok = j < p.L && j >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t rowoff = head + (size_t)min(j, p.L - 1) * D;
  const size_t lbase = (size_t)bh * p.L;

  f32x16 dk[2], dv[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) { dk[0][i] = 0.0f; dk[1][i] = 0.0f; dv[0][i] = 0.0f; dv[1][i] = 0.0f; }
  if (min((J + 1) * BLK, p.L) <= p0) {  // no valid key
    if (j < p.L) {
      store_row_bf16(dK + rowoff, lh, dk, 0.0f, false);
      store_row_bf16(dV + rowoff, lh, dv, 0.0f, false);
    }
    return;
  }
  for (int c = tid; c < 2 * D; c += NT) gate_s[c] = gate_w[(size_t)h * 2 * D + c];
  const float c2 = p.scale * kLog2e;
  bf16x8 kf[4], vf[4];
  load_frags(K + rowoff, lh, c2, kf);
  load_frags(V + rowoff, lh, 1.0f, vf);
  float wv_lt = 0.0f, wv_st = 0.0f;
  if (key_ok) {
    const float2 rc = rowC[lbase + j];
    wv_lt = rc.x;
    wv_st = rc.y;
  }
  float u_lt = 0.0f, u_st = 0.0f;  // sum_i dz[i] P_ij of the two branches (this lane's rows)

  // ---- walk: window part I = J..I_hi, then the inverse selection list ----
  const long last_q = (long)J * BLK + (BLK - 1) + (p.w - 1);
  const int I_hi = (int)min((long)(p.NB - 1), last_q / BLK);
  const int n_st = I_hi - J + 1;
  const int e_lo = offs[(size_t)bh * (p.NB + 1) + J];
  const int n_lt = offs[(size_t)bh * (p.NB + 1) + J + 1] - e_lo;
  const int n_all = n_st + n_lt;
  const int *my_items = items + (size_t)bh * p.NB * p.k + e_lo;
  for (int e = tid; e < min(n_lt, kListRing); e += NT) ring[e] = my_items[e];
  __syncthreads();
  auto tile_of = [&](int t) -> int {  // query block of step t
    return t < n_st ? J + t : __builtin_amdgcn_readfirstlane(ring[(t - n_st) & (kListRing - 1)]);
  };

  Stager<BLK> sg;
  sg.init(wv, lane, p.L, p.NB);
  const int lcol = Stager<BLK>::lane_col(lane);
  const uint16_t *q_lane = Q + head + sg.ld_row * D + lcol;
  const uint16_t *g_lane = dO + head + sg.ld_row * D + lcol;
  const ReadOffsets ro = read_offsets(lane);

  struct RowC { float l2, dox, ax, dz, c0; };
  // per-row constants of query block Iq for one branch (pad rows: probability forced to zero)
  auto row_consts = [&](int Iq, bool windowed) __attribute__((always_inline)) -> RowC {
    RowC r{1.0e30f, 0.0f, 0.0f, 0.0f, 0.0f};
    if (tid < BLK) {
      const int i = Iq * BLK + tid;
      if (i < p.L && i >= p0) {
        const float4 st = rowstat[lbase + i];
        const float4 rb = rowB[lbase + i];
        r.l2 = (windowed ? lse_st[lbase + i] : lse_lt[lbase + i]) * kLog2e;
        r.dox = windowed ? rb.y : rb.x;
        r.ax = windowed ? 1.0f - st.x : st.x;
        r.dz = st.y;
        r.c0 = -st.y * (windowed ? rb.w : rb.z);
      }
    }
    return r;
  };
  auto put_consts = [&](int par, const RowC &r) __attribute__((always_inline)) {
    if (tid < BLK) {
      rc_s[par][0][tid] = r.l2;
      rc_s[par][1][tid] = r.dox;
      rc_s[par][2][tid] = r.ax;
      rc_s[par][3][tid] = r.dz;
      rc_s[par][4][tid] = r.c0;
    }
  };

  auto tile_body = [&](const uint16_t *qs, const uint16_t *gsm, int par, int Iq, bool windowed, float wvx,
                       float &u) __attribute__((always_inline)) {
    const bool masked = windowed || Iq == J || Iq * BLK < p0 || J * BLK < p0 || (Iq + 1) * BLK > p.L;
    // visible <=> key valid and lo_i <= i <= hi_i
    const int lo_i = max(j, p0);
    const int hi_i = windowed ? min(p.L - 1, j + p.w - 1) : p.L - 1;
    const unsigned span = (unsigned)(hi_i - lo_i);
    const bool any = key_ok && hi_i >= lo_i;
#pragma unroll 1
    for (int s = 0; s < UNITS; ++s) {
      f32x16 sacc, gacc;
      const int r0 = 32 * s + 4 * lh;  // this lane's rows of the unit: r0 + 8g + (0..3)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 a = *reinterpret_cast<const float4 *>(&rc_s[par][0][r0 + 8 * g]);
        const float4 b = *reinterpret_cast<const float4 *>(&rc_s[par][1][r0 + 8 * g]);
        sacc[4 * g] = -a.x; sacc[4 * g + 1] = -a.y; sacc[4 * g + 2] = -a.z; sacc[4 * g + 3] = -a.w;
        gacc[4 * g] = -b.x; gacc[4 * g + 1] = -b.y; gacc[4 * g + 2] = -b.z; gacc[4 * g + 3] = -b.w;
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(qs, 32 * s * D + ro.row[kk]), kf[kk], sacc, 0, 0, 0);
        gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(gsm, 32 * s * D + ro.row[kk]), vf[kk], gacc, 0, 0, 0);
      }
      if (masked) {
        const int base = Iq * BLK + 32 * s + 4 * lh;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int qi = base + 8 * (i >> 2) + (i & 3);
          const bool vis = any & ((unsigned)(qi - lo_i) <= span);
          sacc[i] = vis ? sacc[i] : kNegInf;
        }
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 ax4 = *reinterpret_cast<const float4 *>(&rc_s[par][2][r0 + 8 * g]);
        const float4 dz4 = *reinterpret_cast<const float4 *>(&rc_s[par][3][r0 + 8 * g]);
        const float4 c04 = *reinterpret_cast<const float4 *>(&rc_s[par][4][r0 + 8 * g]);
        const float ax[4] = {ax4.x, ax4.y, ax4.z, ax4.w};
        const float dzr[4] = {dz4.x, dz4.y, dz4.z, dz4.w};
        const float c0[4] = {c04.x, c04.y, c04.z, c04.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g + e;
          const float pr = __builtin_amdgcn_exp2f(sacc[i]);
          gacc[i] = pr * fmaf(ax[e], gacc[i], fmaf(dzr[e], wvx, c0[e]));  // dS
          u = fmaf(dzr[e], pr, u);
          sacc[i] = ax[e] * pr;                                            // a_x P
        }
      }
      bf16x8 pf[2], dsf[2];
      to_operand(sacc, pf);
      to_operand(gacc, dsf);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          dv[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(gsm, (32 * s + 16 * t) * D + ro.tr[mb]), pf[t],
                                                           dv[mb], 0, 0, 0);
          dk[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(qs, (32 * s + 16 * t) * D + ro.tr[mb]), dsf[t],
                                                           dk[mb], 0, 0, 0);
        }
      // A probability that is not small (a row with few keys, or a peaked row) multiplies a dO
      // of ordinary size: its bf16 rounding error, 2^-9*P*|dO|, would show in dV, whose other
      // terms are small.  Units holding such a probability add the rounding residuals as a
      // second bf16 term.
      float pmax = sacc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) pmax = fmaxf(pmax, sacc[i]);
      if (__any(pmax > kBigProb)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          sacc[i] -= (float)pf[i >> 3][i & 7];
          gacc[i] -= (float)dsf[i >> 3][i & 7];
        }
        to_operand(sacc, pf);
        to_operand(gacc, dsf);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb) {
            dv[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(gsm, (32 * s + 16 * t) * D + ro.tr[mb]), pf[t],
                                                             dv[mb], 0, 0, 0);
            dk[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(qs, (32 * s + 16 * t) * D + ro.tr[mb]), dsf[t],
                                                             dk[mb], 0, 0, 0);
          }
      }
    }
  };

  {
    const int I0 = tile_of(0);
    sg.stage(q_lane, Qs0, I0);
    sg.stage(g_lane, Gs0, I0);
    put_consts(0, row_consts(I0, 0 < n_st));
  }
  __syncthreads();
  auto step = [&](int t, uint16_t *q_fill, uint16_t *g_fill, const uint16_t *q_cur, const uint16_t *g_cur,
                  int par) __attribute__((always_inline)) {
    RowC rn{1.0e30f, 0.0f, 0.0f, 0.0f, 0.0f};
    const bool more = t + 1 < n_all;
    if (more) {
      const int In = tile_of(t + 1);
      rn = row_consts(In, t + 1 < n_st);
      sg.stage(q_lane, q_fill, In);
      sg.stage(g_lane, g_fill, In);
    }
    // refill the half of the ring that was consumed 64 steps ago
    const int e = t - n_st;
    if (e >= 64 && (e & 63) == 0) {
      const int src = e + 64 + tid;
      if (tid < 64 && src < n_lt) ring[src & (kListRing - 1)] = my_items[src];
    }
    const bool win = t < n_st;
    float u = 0.0f;
    tile_body(q_cur, g_cur, par, tile_of(t), win, win ? wv_st : wv_lt, u);
    u_st += win ? u : 0.0f;
    u_lt += win ? 0.0f : u;
    if (more) put_consts(par ^ 1, rn);
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Qs1, Gs1, Qs0, Gs0, 0);
    if (t + 1 < n_all) step(t + 1, Qs0, Gs0, Qs1, Gs1, 1);
  }
  // rank-one part of dV: Wg_x * sum_i dz[i] P_ij (the other half of the rows sits in lane^32)
  u_lt += __shfl_xor(u_lt, 32);
  u_st += __shfl_xor(u_st, 32);
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int dd = 32 * mb + 8 * (i >> 2) + 4 * lh + (i & 3);
      dv[mb][i] += gate_s[dd] * u_lt + gate_s[D + dd] * u_st;
    }
  if (j < p.L) {
    store_row_bf16(dK + rowoff, lh, dk, p.scale, key_ok);
    store_row_bf16(dV + rowoff, lh, dv, 1.0f, key_ok);
  }
}

bool bwd_mfma_supported(const KParams &p, int dtype)
{
  if (dtype != 1 || p.d != 64 || (p.b != 32 && p.b != 64)) return false;
  return (long)(p.w - 1) / p.b + 2 + p.k <= kMaxTilesQ;
}

void launch_bwd_mfma(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st)
{
  const bool do_dq = stages & kBwdStageDQ, do_dkv = stages & kBwdStageDKV;
  const unsigned grid = (unsigned)(p.B * p.H * p.NB);
  auto u16 = [](const void *x) { return reinterpret_cast<const uint16_t *>(x); };
  if (p.b == 32) {
    if (do_dq) hipLaunchKernelGGL((bwd_dq_mfma_kernel<32>), dim3(grid), dim3(64), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.sel, a.lse_lt, a.lse_st, u16(a.dO), w.rowstat, w.rowB, w.rowC,
                       (uint16_t *)a.dQ, p);
    if (do_dkv) hipLaunchKernelGGL((bwd_dkv_mfma_kernel<32>), dim3(grid), dim3(64), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.gate_w, a.lse_lt, a.lse_st, u16(a.dO), w.rowstat, w.rowB, w.rowC, w.offs,
                       w.items, (uint16_t *)a.dK, (uint16_t *)a.dV, p);
  } else {
    if (do_dq) hipLaunchKernelGGL((bwd_dq_mfma_kernel<64>), dim3(grid), dim3(128), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.sel, a.lse_lt, a.lse_st, u16(a.dO), w.rowstat, w.rowB, w.rowC,
                       (uint16_t *)a.dQ, p);
    if (do_dkv) hipLaunchKernelGGL((bwd_dkv_mfma_kernel<64>), dim3(grid), dim3(128), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.gate_w, a.lse_lt, a.lse_st, u16(a.dO), w.rowstat, w.rowB, w.rowC, w.offs,
                       w.items, (uint16_t *)a.dK, (uint16_t *)a.dV, p);
  }
}

}  // namespace blossom

// Scalar-ALU kernels of the fused attention path for every supported (dtype, d, b):
// forward (both branches + gate, Eq. 1, 16-19), dense causal comparison, and the backward
// pass (gate backward, dQ, inverse selection list, dK/dV, gate-gradient reduction).
//
// Lane mapping: one wavefront per (row, head, block).  A lane owns one row of the block and
// one "phase" of the key (or query) tile: with block size b there are 64/b phases, each
// walking every (64/b)-th row of a tile staged in LDS with its own online-softmax state;
// the phases are merged with wavefront shuffles at the end.  All accumulation is fp32.
// The head dimension (8, 16, 32, 64) is a template parameter; the LDS tiles hold b rows and are
// sized at launch.  With the full short-term mask of Eq. 15 and a mask block smaller than b, the
// far keys of each row (power-of-two distances, last block) are read straight from memory by the
// row's own lanes instead of being walked tile by tile.
#include "common.h"
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

namespace {

constexpr float kNegInf = -__builtin_huge_valf();

template <typename T, int D>
__device__ __forceinline__ void load_row(const T *src, float (&r)[D])
{
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    float x[4];
    load4(src + c, x);
    r[c] = x[0]; r[c + 1] = x[1]; r[c + 2] = x[2]; r[c + 3] = x[3];
  }
}

template <typename T, int D>
__device__ __forceinline__ void store_row(T *dst, const float (&r)[D])
{
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    const float x[4] = {r[c], r[c + 1], r[c + 2], r[c + 3]};
    store4(dst + c, x);
  }
}

// Stage rows [J*b, J*b+b) of one head's [L,D] tensor into LDS as fp32; rows >= L become 0.
template <typename T, int D>
__device__ __forceinline__ void stage_tile(const T *head, int J, int b, int L, float (*dst)[D + 1], int lane)
{
  const int groups = b * (D / 4);
  for (int idx = lane; idx < groups; idx += 64) {
    const int rr = idx / (D / 4);
    const int c4 = (idx % (D / 4)) * 4;
    const int pos = J * b + rr;
    float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (pos < L) load4(head + (size_t)pos * D + c4, x);
    dst[rr][c4] = x[0]; dst[rr][c4 + 1] = x[1]; dst[rr][c4 + 2] = x[2]; dst[rr][c4 + 3] = x[3];
  }
}

__device__ __forceinline__ int first_window_block(int I, int b, int w, int J_first)
{
  const int lowpos = I * b - (w - 1);
  const int J = lowpos <= 0 ? 0 : lowpos / b;
  return J > J_first ? J : J_first;
}

// bidirectional form: last key block the window of a query of block I reaches
__device__ __forceinline__ int last_window_block(int I, int b, int w, int NB)
{
  const long hi = (long)I * b + (b - 1) + (w - 1);
  return (int)min((long)(NB - 1), hi / b);
}

// Far part of the short-term mask when the mask block is smaller than the tile (Eq. 15, second and
// third case, below the window tiles): the rows of a query block then see different, short runs of
// keys, so each lane reads its own keys straight from memory instead of walking whole tiles.
// Calls f(j) once for every key j in [p0, far_hi) at a power-of-two mask-block distance from
// query i, or among the last sblk positions; the runs are dealt over the nph phases of the row.
template <typename F>
__device__ __forceinline__ void far_keys_of_row(const KParams &p, int i, int p0, int far_hi, int phase, int nph, F &&f)
{
  const int qb = i / p.sblk;
  for (int r = phase; r < 31; r += nph) {
    const int mb = qb - (1 << r);
    if (mb < 0) break;
    const int lo = max(mb * p.sblk, p0), hi = min(mb * p.sblk + p.sblk, far_hi);
    for (int j = lo; j < hi; ++j) f(j);
  }
  if (phase == 0)
    for (int j = max(p.last_lo, p0); j < far_hi; ++j)
      if (!is_pow2(qb - j / p.sblk)) f(j);
}
// The same pairs from the key's side: f(i) for every query i in [far_lo, L) that sees key j that way.
template <typename F>
__device__ __forceinline__ void far_rows_of_key(const KParams &p, int j, int far_lo, int phase, int nph, F &&f)
{
  const int kb = j / p.sblk;
  for (int r = phase; r < 31; r += nph) {
    const long first = ((long)kb + (1L << r)) * p.sblk;
    if (first >= p.L) break;
    const int lo = max((int)first, far_lo), hi = min((int)first + p.sblk, p.L);
    for (int i = lo; i < hi; ++i) f(i);
  }
  if (phase == 0 && j >= p.last_lo)
    for (int i = far_lo; i < p.L; ++i)
      if (!is_pow2(i / p.sblk - kb)) f(i);
}
// (host side: picks the instantiation)
// (the bidirectional form walks whole tiles on both sides of the query block)
static inline bool far_by_rows(const KParams &p) { return p.sblk > 0 && p.sblk < p.b && !p.bidir; }

}  // namespace

// =============================================================================================
// Forward
// =============================================================================================
// FAR: the far part of the short-term mask is gathered row by row (mask block smaller than the
// tile); a separate instantiation, so that the plain kernels keep their register budget.
template <typename T, int D, bool FAR>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D <= 32 ? 4 : 2))) void fwd_generic_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                         const T *__restrict__ V,
                                                         const int *__restrict__ valid_len,
                                                         const int *__restrict__ sel,
                                                         const float *__restrict__ gate_w,
                                                         const float *__restrict__ gate_b,
                                                         T *__restrict__ O, float *__restrict__ o_lt_out,
                                                         float *__restrict__ o_st_out,
                                                         float *__restrict__ lse_lt_out,
                                                         float *__restrict__ lse_st_out, int dense,
                                                         KParams p)
{
  // three tiles of b rows (sized at launch: with small blocks a fixed 64-row layout would cap the
  // number of resident wavefronts): K, V, and the short-term output of each row, parked during
  // the long-term pass
  extern __shared__ float fwd_lds[];
  const int lane = threadIdx.x;
  const int b = p.b;
  float (*Ks)[D + 1] = reinterpret_cast<float (*)[D + 1]>(fwd_lds);
  float (*Vs)[D + 1] = Ks + b;
  float (*Os)[D + 1] = Vs + b;
  const int nph = 64 / b;
  const int row = lane % b;
  const int phase = lane / b;
  const int bh = blockIdx.x / p.nq;
  const int I = p.NB - 1 - (int)(blockIdx.x % p.nq);  // late (long) blocks first
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int i = I * b + row;
  const bool in_range = i < p.L;
  const bool active = in_range && i >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t rowoff = head + (size_t)i * D;
  const size_t lrow = (size_t)bh * p.L + i;

  float acc[D];
  if (min((I + 1) * b, p.L) <= p0) {  // no valid query in the block: outputs are zero
    if (phase == 0 && in_range) {
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = 0.0f;
      store_row<T, D>(O + rowoff, acc);
      if (o_lt_out) store_row<float, D>(o_lt_out + rowoff, acc);
      if (o_st_out) store_row<float, D>(o_st_out + rowoff, acc);
      if (lse_lt_out) lse_lt_out[lrow] = 0.0f;
      if (lse_st_out) lse_st_out[lrow] = 0.0f;
    }
    return;
  }

  float q[D];
  if (active) {
    load_row<T, D>(Q + rowoff, q);
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) q[c] = 0.0f;
  }
  const int J_first = p0 / b;
  const T *Kh = K + head;
  const T *Vh = V + head;
  float m, l;

  auto tile = [&](int J, bool windowed) {
    __syncthreads();
    stage_tile<T, D>(Kh, J, b, p.L, Ks, lane);
    stage_tile<T, D>(Vh, J, b, p.L, Vs, lane);
    __syncthreads();
    for (int jj = phase; jj < b; jj += nph) {
      const int j = J * b + jj;
      const bool vis = active && j < p.L && j >= p0 && (j <= i || p.bidir) && (!windowed || st_visible(p, i, j));
      if (vis) {
        float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};  // four independent chains
#pragma unroll
        for (int c = 0; c < D; ++c) s4[c & 3] = fmaf(q[c], Ks[jj][c], s4[c & 3]);
        const float s = ((s4[0] + s4[1]) + (s4[2] + s4[3])) * p.scale;
        if (s > m) {
          const float corr = __expf(m - s);
          l *= corr;
#pragma unroll
          for (int c = 0; c < D; ++c) acc[c] *= corr;
          m = s;
        }
        const float pj = __expf(s - m);
        l += pj;
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] = fmaf(pj, Vs[jj][c], acc[c]);
      }
    }
  };

  auto finish = [&]() -> float {  // merge the phases, normalise; returns lse
    for (int off = b; off < 64; off <<= 1) {
      const float m2 = __shfl_xor(m, off);
      const float l2 = __shfl_xor(l, off);
      const float mn = fmaxf(m, m2);
      const float c1 = (m == kNegInf) ? 0.0f : __expf(m - mn);
      const float c2 = (m2 == kNegInf) ? 0.0f : __expf(m2 - mn);
      l = l * c1 + l2 * c2;
#pragma unroll
      for (int c = 0; c < D; ++c) {
        const float a2 = __shfl_xor(acc[c], off);
        acc[c] = acc[c] * c1 + a2 * c2;
      }
      m = mn;
    }
    float lse = 0.0f;
    if (active) {  // the query itself is always visible, so l > 0
      const float inv = 1.0f / l;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] *= inv;
      lse = m + logf(l);
    } else {
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = 0.0f;
    }
    return lse;
  };

  auto reset = [&]() {
    m = kNegInf;
    l = 0.0f;
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] = 0.0f;
  };

  if (dense) {
    reset();
    for (int J = J_first; J <= I; ++J) tile(J, false);
    const float lse = finish();
    if (phase == 0 && in_range) {
      store_row<T, D>(O + rowoff, acc);
      if (lse_lt_out) lse_lt_out[lrow] = lse;
    }
    return;
  }

  // ---- short-term branch: causal window, plus the keys the other cases of Eq. 15 reach ----
  reset();
  {
    const int J_win = first_window_block(I, b, p.w, J_first);
    if constexpr (FAR) {
      if (active)
        far_keys_of_row(p, i, p0, J_win * b, phase, nph, [&](int j) {
          const T *kp = Kh + (size_t)j * D, *vp = Vh + (size_t)j * D;
          float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float x[4];
            load4(kp + c, x);
#pragma unroll
            for (int e = 0; e < 4; ++e) s4[e] = fmaf(q[c + e], x[e], s4[e]);
          }
          const float s = ((s4[0] + s4[1]) + (s4[2] + s4[3])) * p.scale;
          if (s > m) {
            const float corr = __expf(m - s);
            l *= corr;
#pragma unroll
            for (int c = 0; c < D; ++c) acc[c] *= corr;
            m = s;
          }
          const float pj = __expf(s - m);
          l += pj;
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float x[4];
            load4(vp + c, x);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[c + e] = fmaf(pj, x[e], acc[c + e]);
          }
        });
    } else {
      for (int J = J_first; J < J_win; ++J)
        if (st_block_reach(p, I, J)) tile(J, true);
    }
    for (int J = J_win; J <= I; ++J) tile(J, true);
    if (p.bidir) {  // Eq. 15 as printed: the same on the other side of the query block
      const int J_whi = last_window_block(I, b, p.w, p.NB);
      for (int J = I + 1; J < p.NB; ++J)
        if (J <= J_whi || st_block_reach(p, I, J)) tile(J, true);
    }
  }
  const float lse_st = finish();
  float z = gate_b ? gate_b[h] : 0.0f;
  if (phase == 0) {
    const float *ws = gate_w + (size_t)h * 2 * D + D;
#pragma unroll
    for (int c = 0; c < D; ++c) {
      Os[row][c] = acc[c];
      z = fmaf(ws[c], acc[c], z);
    }
    if (in_range) {
      if (o_st_out) store_row<float, D>(o_st_out + rowoff, acc);
      if (lse_st_out) lse_st_out[lrow] = lse_st;
    }
  }

  // ---- long-term branch: selected blocks ----
  reset();
  const int *my_sel = sel + ((size_t)bh * p.NB + I) * p.k;
  for (int e = 0; e < p.k; ++e) {
    const int J = my_sel[e];
    if (J < 0 || J >= p.NB) continue;
    tile(J, false);
  }
  const float lse_lt = finish();

  // ---- gate and blend (Eq. 18-19) ----
  if (phase == 0 && in_range) {
    if (o_lt_out) store_row<float, D>(o_lt_out + rowoff, acc);
    if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
    const float *wl = gate_w + (size_t)h * 2 * D;
#pragma unroll
    for (int c = 0; c < D; ++c) z = fmaf(wl[c], acc[c], z);
    const float alpha = active ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] = alpha * acc[c] + (1.0f - alpha) * Os[row][c];
    store_row<T, D>(O + rowoff, acc);
  }
}

// =============================================================================================
// Backward, step 1: gate backward per row + per-chunk partial gate-weight gradients.
//   rowstat[row] = (alpha, dz, D_lt, D_st)
//   rowB[row]    = (dO.o_lt, dO.o_st, Wg_lt.o_lt, Wg_st.o_st)      (matrix-core path)
//   rowC[row]    = (Wg_lt.v, Wg_st.v)                               (matrix-core path)
//   partial[(bh*nchunk+chunk)][0..2D] (2D = bias)
// D/4 lanes share a row (16-byte loads, whole rows coalesced), several rows per wavefront step;
// every tensor is read exactly once; the row sums are xor-shuffle reductions over the lanes of
// a row, the gate-weight partials accumulate in registers and meet in LDS in a fixed order.
// =============================================================================================
constexpr int kPrepRows = 128;

template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_prep_kernel(const float *__restrict__ o_lt,
                                                       const float *__restrict__ o_st,
                                                       const T *__restrict__ dO,
                                                       const int *__restrict__ valid_len,
                                                       const float *__restrict__ gate_w,
                                                       const float *__restrict__ gate_b,
                                                       float4 *__restrict__ rowstat,
                                                       float *__restrict__ partial,
                                                       const float *__restrict__ lse_lt,
                                                       const float *__restrict__ lse_st,
                                                       uint16_t *__restrict__ g_lt,
                                                       uint16_t *__restrict__ g_st,
                                                       uint4 *__restrict__ rowI_lt,
                                                       uint4 *__restrict__ rowI_st, KParams p)
{
  constexpr int LPR = D / 4;        // lanes per row
  constexpr int RPW = 64 / LPR;     // rows per wavefront step
  constexpr int RPS = 4 * RPW;      // rows per workgroup step
  constexpr int G = 2 * D + 1;
  __shared__ float red[4 * RPW][G];
  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int sub = lane % LPR, rg = lane / LPR;
  const int c4 = sub * 4;
  const int nchunk = (p.L + kPrepRows - 1) / kPrepRows;
  const int bh = blockIdx.x / nchunk;
  const int chunk = blockIdx.x % nchunk;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const size_t head = (size_t)bh * p.L * D;
  float wl[4], ws[4];
  load4(gate_w + (size_t)h * 2 * D + c4, wl);
  load4(gate_w + (size_t)h * 2 * D + D + c4, ws);
  const float bias = gate_b ? gate_b[h] : 0.0f;
  float acc_l[4] = {0.0f, 0.0f, 0.0f, 0.0f}, acc_s[4] = {0.0f, 0.0f, 0.0f, 0.0f}, acc_b = 0.0f;

  for (int base = 0; base < kPrepRows; base += RPS) {
    const int i = chunk * kPrepRows + base + wave * RPW + rg;
    const bool valid = i < p.L && i >= p0;
    // rows of blocks that hold no valid position are never read by the kernels that follow: nothing is
    // written for them (pad rows of a partly valid block are staged with their tile and get zeros)
    const bool inb = i < p.L && i >= (p0 / p.b) * p.b;
    float g[4] = {0.f, 0.f, 0.f, 0.f}, ol[4] = {0.f, 0.f, 0.f, 0.f}, os[4] = {0.f, 0.f, 0.f, 0.f};
    if (valid) {
      const size_t ro = head + (size_t)i * D + c4;
      load4(dO + ro, g);
      load4(o_lt + ro, ol);
      load4(o_st + ro, os);
    }
    float a_ll = 0.f, a_ss = 0.f, w_l = 0.f, w_s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a_ll = fmaf(g[e], ol[e], a_ll);
      a_ss = fmaf(g[e], os[e], a_ss);
      w_l = fmaf(wl[e], ol[e], w_l);
      w_s = fmaf(ws[e], os[e], w_s);
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) {
      a_ll += __shfl_xor(a_ll, off);
      a_ss += __shfl_xor(a_ss, off);
      w_l += __shfl_xor(w_l, off);
      w_s += __shfl_xor(w_s, off);
    }
    float4 st = make_float4(0.f, 0.f, 0.f, 0.f);
    float dz = 0.0f, alpha = 0.0f;
    if (valid) {
      const float z = bias + w_l + w_s;
      alpha = 1.0f / (1.0f + __expf(-z));
      dz = (a_ll - a_ss) * alpha * (1.0f - alpha);
      st = make_float4(alpha, dz, alpha * a_ll + dz * w_l, (1.0f - alpha) * a_ss + dz * w_s);
    }
    if (inb && sub == 0) rowstat[(size_t)bh * p.L + i] = st;
    if (g_lt) {
      // Matrix-core path: the upstream gradient of each branch, dO_x = a_x*dO + dz*Wg_x, rounded
      // to bf16 once, and the row constant c_x = dO_x.o_x taken with the SAME rounded values, so
      // that P*(dO_x.v - c_x) is the exact softmax backward of the rounded gradient (rows with a
      // single key still cancel to zero).  -lse*log2(e) and -c_x are left as three-term bf16
      // splits, the form in which one matrix instruction broadcasts them into an accumulator.
      uint16_t gl[4], gs[4];
      float c_l = 0.0f, c_s = 0.0f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        gl[e] = f32_to_bf16(fmaf(alpha, g[e], dz * wl[e]));
        gs[e] = f32_to_bf16(fmaf(1.0f - alpha, g[e], dz * ws[e]));
        c_l = fmaf(bf16_to_f32(gl[e]), ol[e], c_l);
        c_s = fmaf(bf16_to_f32(gs[e]), os[e], c_s);
      }
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) {
        c_l += __shfl_xor(c_l, off);
        c_s += __shfl_xor(c_s, off);
      }
      if (inb) {
        const size_t ro = head + (size_t)i * D + c4;
        *reinterpret_cast<uint2 *>(g_lt + ro) =
            make_uint2((uint32_t)gl[0] | ((uint32_t)gl[1] << 16), (uint32_t)gl[2] | ((uint32_t)gl[3] << 16));
        *reinterpret_cast<uint2 *>(g_st + ro) =
            make_uint2((uint32_t)gs[0] | ((uint32_t)gs[1] << 16), (uint32_t)gs[2] | ((uint32_t)gs[3] << 16));
        if (sub == 0) {
          const size_t r = (size_t)bh * p.L + i;
          // pad rows: an exponent of -1e30 makes every probability of the row zero
          const uint2 l_l = mfma::split3(valid ? -lse_lt[r] * 1.4426950408889634f : -1.0e30f);
          const uint2 l_s = mfma::split3(valid ? -lse_st[r] * 1.4426950408889634f : -1.0e30f);
          const uint2 k_l = mfma::split3(-c_l), k_s = mfma::split3(-c_s);
          rowI_lt[r] = make_uint4(l_l.x, l_l.y, k_l.x, k_l.y);
          rowI_st[r] = make_uint4(l_s.x, l_s.y, k_s.x, k_s.y);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc_l[e] = fmaf(dz, ol[e], acc_l[e]);
      acc_s[e] = fmaf(dz, os[e], acc_s[e]);
    }
    acc_b += dz;
  }
  const int slot = wave * RPW + rg;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    red[slot][c4 + e] = acc_l[e];
    red[slot][D + c4 + e] = acc_s[e];
  }
  if (sub == 0) red[slot][2 * D] = acc_b;
  __syncthreads();
  float *out = partial + (size_t)blockIdx.x * G;
  for (int c = t; c < G; c += 256) {
    float acc = 0.0f;
#pragma unroll
    for (int sl = 0; sl < 4 * RPW; ++sl) acc += red[sl][c];
    out[c] = acc;
  }
}

// Fixed-order reduction of the partial gate gradients over batch rows and chunks, two levels:
// level 1 sums kGateSlices contiguous slices of a head's partials, level 2 sums the slices.
constexpr int kGateSlices = 32;

__global__ __launch_bounds__(256) void bwd_gate_reduce1_kernel(const float *__restrict__ partial,
                                                               float *__restrict__ stage2, int nchunk, KParams p)
{
  const int h = blockIdx.x;
  const int sl = blockIdx.y;
  const int G = 2 * p.d + 1;
  const int N = p.B * nchunk;  // partial rows of this head, ordered by (batch row, chunk)
  const int per = (N + kGateSlices - 1) / kGateSlices;
  const int lo = sl * per, hi = min(N, lo + per);
  // one thread per output column; four independent running sums keep four loads in flight, and
  // are added in a fixed order at the end
  for (int c = threadIdx.x; c < G; c += blockDim.x) {
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    auto at = [&](int nn) -> float {
      const int r = nn / nchunk, ch = nn % nchunk;
      return partial[(((size_t)r * p.H + h) * nchunk + ch) * G + c];
    };
    int nn = lo;
    for (; nn + 4 <= hi; nn += 4) {
      const float v0 = at(nn), v1 = at(nn + 1), v2 = at(nn + 2), v3 = at(nn + 3);
      acc[0] += v0; acc[1] += v1; acc[2] += v2; acc[3] += v3;
    }
    for (; nn < hi; ++nn) acc[0] += at(nn);
    stage2[((size_t)h * kGateSlices + sl) * G + c] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  }
}

__global__ __launch_bounds__(256) void bwd_gate_reduce2_kernel(const float *__restrict__ stage2,
                                                               float *__restrict__ d_gate_w,
                                                               float *__restrict__ d_gate_b, KParams p)
{
  const int h = blockIdx.x;
  const int G = 2 * p.d + 1;
  for (int c = threadIdx.x; c < G; c += blockDim.x) {
    float acc = 0.0f;
    for (int sl = 0; sl < kGateSlices; ++sl) acc += stage2[((size_t)h * kGateSlices + sl) * G + c];
    if (c < 2 * p.d) d_gate_w[(size_t)h * 2 * p.d + c] = acc;
    else if (d_gate_b) d_gate_b[h] = acc;
  }
}

// =============================================================================================
// Backward, step 2: dQ (query-block stationary, same tile walk as the forward).
//   dP_ij = dO_x[i].v_j = a_x[i]*(dO[i].v_j) + dz[i]*(gate_w_x.v_j)
// =============================================================================================
template <typename T, int D, bool FAR>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(D <= 32 ? 3 : 1))) void bwd_dq_generic_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                            const T *__restrict__ V,
                                                            const int *__restrict__ valid_len,
                                                            const int *__restrict__ sel,
                                                            const float *__restrict__ gate_w,
                                                            const float *__restrict__ lse_lt,
                                                            const float *__restrict__ lse_st,
                                                            const T *__restrict__ dO,
                                                            const float4 *__restrict__ rowstat,
                                                            T *__restrict__ dQ, KParams p)
{
  extern __shared__ float dq_lds[];  // K and V tiles of b rows (sized at launch)
  __shared__ float wv[64];           // gate_w_x . v_j of the staged tile

  const int lane = threadIdx.x;
  const int b = p.b;
  float (*Ks)[D + 1] = reinterpret_cast<float (*)[D + 1]>(dq_lds);
  float (*Vs)[D + 1] = Ks + b;
  const int nph = 64 / b;
  const int row = lane % b;
  const int phase = lane / b;
  const int bh = blockIdx.x / p.NB;
  const int I = p.NB - 1 - (int)(blockIdx.x % p.NB);
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int i = I * b + row;
  const bool in_range = i < p.L;
  const bool active = in_range && i >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t rowoff = head + (size_t)i * D;

  float dq[D];
#pragma unroll
  for (int c = 0; c < D; ++c) dq[c] = 0.0f;
  if (min((I + 1) * b, p.L) <= p0) {
    if (phase == 0 && in_range) store_row<T, D>(dQ + rowoff, dq);
    return;
  }
  float q[D], g[D];
  float4 st = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  float l_lt = 0.0f, l_st = 0.0f;
  if (active) {
    load_row<T, D>(Q + rowoff, q);
    load_row<T, D>(dO + rowoff, g);
    st = rowstat[(size_t)bh * p.L + i];
    l_lt = lse_lt[(size_t)bh * p.L + i];
    l_st = lse_st[(size_t)bh * p.L + i];
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) { q[c] = 0.0f; g[c] = 0.0f; }
  }
  const int J_first = p0 / b;
  const T *Kh = K + head;
  const T *Vh = V + head;

  auto tile = [&](int J, bool windowed) {
    const float *wx = gate_w + (size_t)h * 2 * D + (windowed ? D : 0);
    const float a_x = windowed ? 1.0f - st.x : st.x;
    const float D_x = windowed ? st.w : st.z;
    const float lse = windowed ? l_st : l_lt;
    __syncthreads();
    stage_tile<T, D>(Kh, J, b, p.L, Ks, lane);
    stage_tile<T, D>(Vh, J, b, p.L, Vs, lane);
    __syncthreads();
    if (lane < b) {
      float a = 0.0f;
      for (int c = 0; c < D; ++c) a = fmaf(wx[c], Vs[lane][c], a);
      wv[lane] = a;
    }
    __syncthreads();
    for (int jj = phase; jj < b; jj += nph) {
      const int j = J * b + jj;
      const bool vis = active && j < p.L && j >= p0 && (j <= i || p.bidir) && (!windowed || st_visible(p, i, j));
      if (vis) {
        float s = 0.0f, gv = 0.0f;
#pragma unroll
        for (int c = 0; c < D; ++c) {
          s = fmaf(q[c], Ks[jj][c], s);
          gv = fmaf(g[c], Vs[jj][c], gv);
        }
        const float pj = __expf(s * p.scale - lse);
        const float dS = pj * (a_x * gv + st.y * wv[jj] - D_x);
#pragma unroll
        for (int c = 0; c < D; ++c) dq[c] = fmaf(dS, Ks[jj][c], dq[c]);
      }
    }
  };

  {
    const int J_win = first_window_block(I, b, p.w, J_first);
    if constexpr (FAR) {
      const float *wx = gate_w + (size_t)h * 2 * D + D;
      if (active)
        far_keys_of_row(p, i, p0, J_win * b, phase, nph, [&](int j) {
          const T *kp = Kh + (size_t)j * D, *vp = Vh + (size_t)j * D;
          float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, g4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, w4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float kx[4], vx[4];
            load4(kp + c, kx);
            load4(vp + c, vx);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              s4[e] = fmaf(q[c + e], kx[e], s4[e]);
              g4[e] = fmaf(g[c + e], vx[e], g4[e]);
              w4[e] = fmaf(wx[c + e], vx[e], w4[e]);
            }
          }
          const float sj = (s4[0] + s4[1]) + (s4[2] + s4[3]);
          const float gv = (g4[0] + g4[1]) + (g4[2] + g4[3]);
          const float wvj = (w4[0] + w4[1]) + (w4[2] + w4[3]);
          const float pj = __expf(sj * p.scale - l_st);
          const float dS = pj * ((1.0f - st.x) * gv + st.y * wvj - st.w);
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float kx[4];
            load4(kp + c, kx);
#pragma unroll
            for (int e = 0; e < 4; ++e) dq[c + e] = fmaf(dS, kx[e], dq[c + e]);
          }
        });
    } else {
      for (int J = J_first; J < J_win; ++J)
        if (st_block_reach(p, I, J)) tile(J, true);
    }
    for (int J = J_win; J <= I; ++J) tile(J, true);
    if (p.bidir) {  // Eq. 15 as printed: the same on the other side of the query block
      const int J_whi = last_window_block(I, b, p.w, p.NB);
      for (int J = I + 1; J < p.NB; ++J)
        if (J <= J_whi || st_block_reach(p, I, J)) tile(J, true);
    }
  }
  const int *my_sel = sel + ((size_t)bh * p.NB + I) * p.k;
  for (int e = 0; e < p.k; ++e) {
    const int J = my_sel[e];
    if (J < 0 || J >= p.NB) continue;
    tile(J, false);
  }
  for (int off = b; off < 64; off <<= 1) {
#pragma unroll
    for (int c = 0; c < D; ++c) dq[c] += __shfl_xor(dq[c], off);
  }
  if (phase == 0 && in_range) {
#pragma unroll
    for (int c = 0; c < D; ++c) dq[c] *= p.scale;
    unrope_row<D>(p, i, dq);
    store_row<T, D>(dQ + rowoff, dq);
  }
}

// =============================================================================================
// Backward, step 3: inverse selection list.  For each key block J of a (row, head): the list of
// query blocks I whose selection holds J, in a fixed, deterministic order.
// offs [B*H,(NB+1)], items [B*H,NB*k].
// One workgroup of W wavefronts per (row, head); wavefront w owns a contiguous range of query
// blocks and its own counters.  Counting and filling use LDS integer atomics, one selection
// row per wavefront instruction: a row lists distinct blocks, and the LDS executes one
// wavefront's instructions in order, so the order inside a wavefront's range is that of the
// fill loop: by 64-entry chunk of the selection row, then by I (ascending in I whenever
// topk <= 64); the ranges are laid out one after the other per key block (the scan hands each
// wavefront its base).  The consumers sum over the list and need no particular order, only the
// same one on every run.
// =============================================================================================
constexpr int kInvWaves = 4;      // wavefronts per (row, head) when the counters fit
constexpr int kInvWavesMaxNB = 2048;

__global__ __launch_bounds__(64 * kInvWaves) void inverse_list_kernel(const int *__restrict__ sel,
                                                                      const int *__restrict__ valid_len,
                                                                      int *__restrict__ offs, int *__restrict__ items,
                                                                      KParams p)
{
  extern __shared__ int inv_lds[];  // cnt[W][NB+1], then few[NB+1] bytes
  const int W = blockDim.x >> 6;
  const int stride = p.NB + 1;
  int *cnt = inv_lds;
  unsigned char *few = reinterpret_cast<unsigned char *>(inv_lds + W * stride);  // query block whose selected
                                                                                  // past blocks hold few valid keys
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = tid >> 6;
  const int bh = blockIdx.x;
  const int *s = sel + (size_t)bh * p.NB * p.k;
  int *o = offs + (size_t)bh * (p.NB + 1);
  int *it = items + (size_t)bh * p.NB * p.k;
  const int p0 = p.L - clamp_len(valid_len[bh / p.H], p.L);
  const int per = (p.NB + W - 1) / W;
  const int I_lo = wv * per, I_hi = min(p.NB, I_lo + per);
  int *mine = cnt + wv * stride;
  for (int x = tid; x < W * stride; x += blockDim.x) cnt[x] = 0;
  for (int J = tid; J <= p.NB; J += blockDim.x) few[J] = 1;
  __syncthreads();
  for (int e0 = 0; e0 < p.k; e0 += 64) {
    const int e = e0 + lane;
#pragma unroll 8
    for (int I = I_lo; I < I_hi; ++I) {
      const int J = e < p.k ? s[(size_t)I * p.k + e] : -1;
      if (J >= 0 && J < p.NB && (J <= I || p.bidir)) atomicAdd(&mine[J], 1);
      // an earlier block with at least kInvFewKeys valid keys gives every row of I that many keys
      const int vcount = min((J + 1) * p.b, p.L) - max(J * p.b, p0);
      if (__ballot(J >= 0 && J < I && vcount >= kInvFewKeys) != 0ull && lane == 0) few[I] = 0;
    }
  }
  __syncthreads();
  // exclusive scan over (key block, wavefront) in chunks of 64 key blocks; o[NB] receives the total
  if (wv == 0) {
    int carry = 0;
    for (int J0 = 0; J0 <= p.NB; J0 += 64) {
      const int J = J0 + lane;
      int c = 0;
      if (J < p.NB)
        for (int w = 0; w < W; ++w) c += cnt[w * stride + J];
      int incl = c;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
      }
      if (J <= p.NB) {
        int base = carry + incl - c;
        o[J] = base;
        if (J < p.NB)
          for (int w = 0; w < W; ++w) {
            const int cw = cnt[w * stride + J];
            cnt[w * stride + J] = base;
            base += cw;
          }
      }
      carry += __shfl(incl, 63);
    }
  }
  __syncthreads();
  for (int e0 = 0; e0 < p.k; e0 += 64) {
    const int e = e0 + lane;
#pragma unroll 8
    for (int I = I_lo; I < I_hi; ++I) {
      const int J = e < p.k ? s[(size_t)I * p.k + e] : -1;
      if (J >= 0 && J < p.NB && (J <= I || p.bidir)) it[atomicAdd(&mine[J], 1)] = I | ((int)few[I] << kInvFewShift);
    }
  }
}

// =============================================================================================
// Backward, step 4: dK / dV (key-block stationary).  MODE 0 computes dV, 1 dK, 2 both.  With
// d >= 32 they are one launch each: the dV pass needs neither the V row nor the dP product, so it
// runs with fewer registers and more wavefronts; with small d one pass holds both.
// A lane owns one key row and one phase of the query tile.
// =============================================================================================
template <typename T, int D, int MODE, bool FAR>
__global__ __launch_bounds__(64) void bwd_dkv_generic_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                             const T *__restrict__ V,
                                                             const int *__restrict__ valid_len,
                                                             const float *__restrict__ gate_w,
                                                             const float *__restrict__ lse_lt,
                                                             const float *__restrict__ lse_st,
                                                             const T *__restrict__ dO,
                                                             const float4 *__restrict__ rowstat,
                                                             const int *__restrict__ offs,
                                                             const int *__restrict__ items,
                                                             T *__restrict__ dK, T *__restrict__ dV,
                                                             KParams p)
{
  extern __shared__ float dkv_lds[];  // Q and dO_x tiles of b rows (sized at launch)
  __shared__ float lse_s[64];
  __shared__ float Dx_s[64];

  const int lane = threadIdx.x;
  const int b = p.b;
  float (*Qs)[D + 1] = reinterpret_cast<float (*)[D + 1]>(dkv_lds);
  float (*Gs)[D + 1] = Qs + b;  // dO_x rows of the staged query tile
  const int nph = 64 / b;
  const int jj = lane % b;
  const int phase = lane / b;
  const int bh = blockIdx.x / p.NB;
  const int J = (int)(blockIdx.x % p.NB);
  constexpr bool want_dk = MODE != 0, want_dv = MODE != 1;
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int j = J * b + jj;
  const bool in_range = j < p.L;
  const bool key_ok = in_range && j >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t outoff = head + (size_t)j * D;

  float acck[D], accv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { acck[c] = 0.0f; accv[c] = 0.0f; }
  if (min((J + 1) * b, p.L) <= p0) {  // no valid key in the block
    if (phase == 0 && in_range) {
      if (want_dk) store_row<T, D>(dK + outoff, acck);
      if (want_dv) store_row<T, D>(dV + outoff, accv);
    }
    return;
  }
  float kr[D], vr[D];
  if (key_ok) {
    load_row<T, D>(K + head + (size_t)j * D, kr);
    if (want_dk) load_row<T, D>(V + head + (size_t)j * D, vr);
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) { kr[c] = 0.0f; vr[c] = 0.0f; }
  }
  const T *Qh = Q + head;
  const T *Gh = dO + head;

  auto tile = [&](int I, bool windowed) {
    const float *wx = gate_w + (size_t)h * 2 * D + (windowed ? D : 0);
    __syncthreads();
    stage_tile<T, D>(Qh, I, b, p.L, Qs, lane);
    // dO_x = a_x*dO + dz*gate_w_x, formed while staging
    const int groups = b * (D / 4);
    for (int idx = lane; idx < groups; idx += 64) {
      const int rr = idx / (D / 4);
      const int c4 = (idx % (D / 4)) * 4;
      const int pos = I * b + rr;
      float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (pos < p.L && pos >= p0) {
        load4(Gh + (size_t)pos * D + c4, x);
        const float4 st = rowstat[(size_t)bh * p.L + pos];
        const float a_x = windowed ? 1.0f - st.x : st.x;
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = a_x * x[e] + st.y * wx[c4 + e];
      }
      Gs[rr][c4] = x[0]; Gs[rr][c4 + 1] = x[1]; Gs[rr][c4 + 2] = x[2]; Gs[rr][c4 + 3] = x[3];
    }
    if (lane < b) {
      const int pos = I * b + lane;
      float l = 0.0f, dx = 0.0f;
      if (pos < p.L && pos >= p0) {
        const float4 st = rowstat[(size_t)bh * p.L + pos];
        l = windowed ? lse_st[(size_t)bh * p.L + pos] : lse_lt[(size_t)bh * p.L + pos];
        dx = windowed ? st.w : st.z;
      }
      lse_s[lane] = l;
      Dx_s[lane] = dx;
    }
    __syncthreads();
    for (int ii = phase; ii < b; ii += nph) {
      const int i = I * b + ii;
      const bool vis = key_ok && i < p.L && i >= p0 && (j <= i || p.bidir) && (!windowed || st_visible(p, i, j));
      if (vis) {
        float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};  // four independent chains
#pragma unroll
        for (int c = 0; c < D; ++c) s4[c & 3] = fmaf(Qs[ii][c], kr[c], s4[c & 3]);
        const float s = (s4[0] + s4[1]) + (s4[2] + s4[3]);
        const float pj = __expf(s * p.scale - lse_s[ii]);
        if (want_dk) {
          float d4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int c = 0; c < D; ++c) d4[c & 3] = fmaf(Gs[ii][c], vr[c], d4[c & 3]);
          const float dP = (d4[0] + d4[1]) + (d4[2] + d4[3]);
          const float dS = pj * (dP - Dx_s[ii]);
#pragma unroll
          for (int c = 0; c < D; ++c) acck[c] = fmaf(dS, Qs[ii][c], acck[c]);
        }
        if (want_dv) {
#pragma unroll
          for (int c = 0; c < D; ++c) accv[c] = fmaf(pj, Gs[ii][c], accv[c]);
        }
      }
    }
  };

  // short-term branch: query blocks whose window reaches this key block, then those that
  // reach it through the other cases of Eq. 15
  {
    const long last_q = (long)J * b + (b - 1) + (p.w - 1);
    const int I_hi = (int)min((long)(p.NB - 1), last_q / b);
    for (int I = J; I <= I_hi; ++I) tile(I, true);
    if (p.bidir) {  // query blocks before the key block: window reach, then the other cases of Eq. 15
      const int I_first = p0 / b;
      const int I_lo = first_window_block(J, b, p.w, I_first);
      for (int I = I_first; I < J; ++I)
        if (I >= I_lo || st_block_reach(p, I, J)) tile(I, true);
    }
    if constexpr (FAR) {
      const float *wx = gate_w + (size_t)h * 2 * D + D;
      if (key_ok)
        far_rows_of_key(p, j, (I_hi + 1) * b, phase, nph, [&](int i) {
          const size_t r = (size_t)bh * p.L + i;
          const float4 st = rowstat[r];
          const float a_x = 1.0f - st.x;
          const T *qp = Qh + (size_t)i * D, *gp = Gh + (size_t)i * D;
          float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float qx[4];
            load4(qp + c, qx);
#pragma unroll
            for (int e = 0; e < 4; ++e) s4[e] = fmaf(qx[e], kr[c + e], s4[e]);
          }
          const float pj = __expf(((s4[0] + s4[1]) + (s4[2] + s4[3])) * p.scale - lse_st[r]);
          float d4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int c = 0; c < D; c += 4) {
            float gx[4];
            load4(gp + c, gx);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float gxe = a_x * gx[e] + st.y * wx[c + e];  // dO_st
              if (want_dk) d4[e] = fmaf(gxe, vr[c + e], d4[e]);
              if (want_dv) accv[c + e] = fmaf(pj, gxe, accv[c + e]);
            }
          }
          if (want_dk) {
            const float dS = pj * (((d4[0] + d4[1]) + (d4[2] + d4[3])) - st.w);
#pragma unroll
            for (int c = 0; c < D; c += 4) {
              float qx[4];
              load4(qp + c, qx);
#pragma unroll
              for (int e = 0; e < 4; ++e) acck[c + e] = fmaf(dS, qx[e], acck[c + e]);
            }
          }
        });
    } else {
      for (int I = I_hi + 1; I < p.NB; ++I)
        if (st_block_reach(p, I, J)) tile(I, true);
    }
  }
  // long-term branch: query blocks that selected this key block
  {
    const int *o = offs + (size_t)bh * (p.NB + 1);
    const int *it = items + (size_t)bh * p.NB * p.k;
    const int e_lo = o[J], e_hi = o[J + 1];
    for (int e = e_lo; e < e_hi; ++e) tile(it[e] & kInvBlockMask, false);
  }
  for (int off = b; off < 64; off <<= 1) {
#pragma unroll
    for (int c = 0; c < D; ++c) {
      if (want_dk) acck[c] += __shfl_xor(acck[c], off);
      if (want_dv) accv[c] += __shfl_xor(accv[c], off);
    }
  }
  if (phase == 0 && in_range) {
    if (want_dk) {
#pragma unroll
      for (int c = 0; c < D; ++c) acck[c] *= p.scale;
      unrope_row<D>(p, j, acck);
      store_row<T, D>(dK + outoff, acck);
    }
    if (want_dv) store_row<T, D>(dV + outoff, accv);
  }
}

// =============================================================================================
// Launchers
// =============================================================================================
template <typename T, int D>
static void launch_fwd_t(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3((unsigned)(p.B * p.H * p.nq)), dim3(64),
                       3 * (size_t)p.b * (D + 1) * sizeof(float), st,
                       (const T *)a.Q, (const T *)a.K, (const T *)a.V, a.valid_len, a.sel, a.gate_w,
                       a.gate_b, (T *)a.O, (float *)a.o_lt, (float *)a.o_st, a.lse_lt, a.lse_st, a.dense, p);
  };
  if (far_by_rows(p) && !a.dense) go(fwd_generic_kernel<T, D, true>);
  else go(fwd_generic_kernel<T, D, false>);
}

void launch_fwd_generic(const KParams &p, int dtype, const FwdArgs &a, hipStream_t st)
{
  with_head_dim(p.d, [&](auto dim) {
    constexpr int D = decltype(dim)::value;
    if (dtype == 0) launch_fwd_t<float, D>(p, a, st);
    else launch_fwd_t<bf16_t, D>(p, a, st);
  });
}

namespace {
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
}  // namespace

BwdWorkspace bwd_carve(const KParams &p, int dtype, void *ws)
{
  BwdWorkspace w{};
  char *base = reinterpret_cast<char *>(ws);
  const size_t BH = (size_t)p.B * p.H;
  w.nchunk = (p.L + kPrepRows - 1) / kPrepRows;
  size_t off = 0;
  w.rowstat = reinterpret_cast<float4 *>(base + off);
  off = align256(off + BH * p.L * sizeof(float4));
  w.offs = reinterpret_cast<int *>(base + off);
  off = align256(off + BH * (p.NB + 1) * sizeof(int));
  w.items = reinterpret_cast<int *>(base + off);
  off = align256(off + BH * p.NB * p.k * sizeof(int));
  w.partial = reinterpret_cast<float *>(base + off);
  off = align256(off + BH * w.nchunk * (2 * p.d + 1) * sizeof(float));
  w.stage2 = reinterpret_cast<float *>(base + off);
  off = align256(off + (size_t)p.H * kGateSlices * (2 * p.d + 1) * sizeof(float));
  if (bwd_mfma_supported(p, dtype)) {
    w.g_lt = reinterpret_cast<uint16_t *>(base + off);
    off = align256(off + BH * p.L * p.d * sizeof(uint16_t));
    w.g_st = reinterpret_cast<uint16_t *>(base + off);
    off = align256(off + BH * p.L * p.d * sizeof(uint16_t));
    w.rowI_lt = reinterpret_cast<uint4 *>(base + off);
    off = align256(off + BH * p.L * sizeof(uint4));
    w.rowI_st = reinterpret_cast<uint4 *>(base + off);
    off = align256(off + BH * p.L * sizeof(uint4));
  }
  w.total = off;
  return w;
}

size_t bwd_workspace_bytes(const KParams &p, int dtype) { return bwd_carve(p, dtype, nullptr).total; }

template <typename T, int D>
static void launch_bwd_t(const KParams &p, int dtype, const BwdArgs &a, unsigned stages, hipStream_t st)
{
  const BwdWorkspace w = bwd_carve(p, dtype, a.ws);
  const unsigned BH = (unsigned)(p.B * p.H);
  const bool mfma = bwd_mfma_supported(p, dtype);

  if (stages & kBwdStageGate) {
    BLOSSOM_LAUNCH((bwd_prep_kernel<T, D>), dim3(BH * w.nchunk), dim3(256), 0, st,
                       (const float *)a.o_lt, (const float *)a.o_st, (const T *)a.dO, a.valid_len, a.gate_w,
                       a.gate_b, w.rowstat, w.partial, a.lse_lt, a.lse_st, w.g_lt, w.g_st, w.rowI_lt, w.rowI_st, p);
    BLOSSOM_LAUNCH(bwd_gate_reduce1_kernel, dim3((unsigned)p.H, kGateSlices), dim3(256), 0, st, w.partial,
                       w.stage2, w.nchunk, p);
    BLOSSOM_LAUNCH(bwd_gate_reduce2_kernel, dim3((unsigned)p.H), dim3(256), 0, st, w.stage2, a.d_gate_w,
                       a.d_gate_b, p);
  }
  if (stages & kBwdStageInverse) {
    const int W = p.NB <= kInvWavesMaxNB ? kInvWaves : 1;
    const size_t lds = (size_t)W * (p.NB + 1) * sizeof(int) + (size_t)(p.NB + 1 + 3) / 4 * 4;
    BLOSSOM_LAUNCH(inverse_list_kernel, dim3(BH), dim3(64 * W), lds, st, a.sel, a.valid_len, w.offs, w.items,
                       p);
  }
  if (mfma) {
    if (launch_failed()) return;
    launch_bwd_mfma(p, a, w, stages, st);
    return;
  }
  if (bwd_res_supported(p, dtype)) {
    if (launch_failed()) return;
    launch_bwd_res(p, dtype, a, w, stages, st);
    return;
  }
  const size_t lds = 2 * (size_t)p.b * (D + 1) * sizeof(float);  // two tiles of b rows
  const bool far = far_by_rows(p);
  if (stages & kBwdStageDQ) {
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(BH * p.NB), dim3(64), lds, st, (const T *)a.Q, (const T *)a.K,
                         (const T *)a.V, a.valid_len, a.sel, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO,
                         w.rowstat, (T *)a.dQ, p);
    };
    if (far) go(bwd_dq_generic_kernel<T, D, true>);
    else go(bwd_dq_generic_kernel<T, D, false>);
    if (launch_failed()) return;
  }
  if (stages & kBwdStageDKV) {
    auto go = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(BH * p.NB), dim3(64), lds, st, (const T *)a.Q, (const T *)a.K,
                         (const T *)a.V, a.valid_len, a.gate_w, a.lse_lt, a.lse_st, (const T *)a.dO, w.rowstat,
                         w.offs, w.items, (T *)a.dK, (T *)a.dV, p);
    };
    if constexpr (D <= 16) {
      if (far) go(bwd_dkv_generic_kernel<T, D, 2, true>);
      else go(bwd_dkv_generic_kernel<T, D, 2, false>);
    } else {
      if (far) {
        go(bwd_dkv_generic_kernel<T, D, 0, true>);
        if (launch_failed()) return;
        go(bwd_dkv_generic_kernel<T, D, 1, true>);
      } else {
        go(bwd_dkv_generic_kernel<T, D, 0, false>);
        if (launch_failed()) return;
        go(bwd_dkv_generic_kernel<T, D, 1, false>);
      }
    }
  }
}

void launch_bwd(const KParams &p, int dtype, const BwdArgs &a, unsigned stages, hipStream_t st)
{
  with_head_dim(p.d, [&](auto dim) {
    constexpr int D = decltype(dim)::value;
    if (dtype == 0) launch_bwd_t<float, D>(p, dtype, a, stages, st);
    else launch_bwd_t<bf16_t, D>(p, dtype, a, stages, st);
  });
}

}  // namespace blossom

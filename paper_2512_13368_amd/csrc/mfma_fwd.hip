// Fused forward on the matrix cores for bf16, d = 64, block size 32 or 64 (Eq. 1 under the two
// branch masks, Eq. 16-19), plus the same-style dense causal comparison.
//
// Work split: one workgroup per (row, head, query block); one wavefront per 32 query rows.
// K/V tiles of the short-term window and of the selected blocks are gathered by the selection
// list from HBM/L2 with coalesced 16-byte loads, staged in LDS (double buffered) and shared by
// the workgroup's wavefronts.
//
// Per 32-key sub-tile a wavefront computes S^T = K Q^T with four v_mfma_f32_32x32x16_bf16
// (keys are the M dimension, so every lane owns ONE query column and 16 of its logits: the
// row maximum and row sum are in-lane reductions plus one exchange with lane^32), applies the
// online softmax in fp32, and feeds P^T straight from the accumulator registers (converted to
// bf16) as the B operand of O^T += V^T P^T (four more MFMAs).  The key order inside a
// contraction slab is whatever the accumulator layout dictates; V^T is read from LDS with the
// transposing ds_read_b64_tr_b16 in exactly that order, so P never moves between lanes.
#include "common.h"
#include "launch.h"

namespace blossom {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = 64;
constexpr int KSTR = 72;  // bf16 elements per K row in LDS: 144 B, conflict-free 16-byte row reads
constexpr int VSTR = 80;  // 160 B rows for the 4-row x 32-byte patches of the transposing read
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegInf = -__builtin_huge_valf();

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Maps the hardware workgroup id (dealt round-robin over the 8 XCDs) to a virtual id such that
// each XCD works through a contiguous range: all query blocks of a head then share one L2.
__device__ __forceinline__ unsigned xcd_remap(unsigned pid, unsigned total)
{
  constexpr unsigned X = 8;
  const unsigned per = (total + X - 1) / X;      // ids of a "tall" XCD
  const unsigned tall = total % X ? total % X : X;
  const unsigned xcd = pid % X, local = pid / X;
  return xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
}

struct Tile16 {  // one thread's share of a staged K or V tile: 4 x 16 bytes
  uint4 r[4];
};

template <int BLK>
__device__ __forceinline__ void tile_load(const uint16_t *head, int J, int L, int tid, Tile16 &t)
{
  constexpr int NT = BLK * 2;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int c = tid + NT * u;
    const int row = c >> 3, col = c & 7;
    const int pos = J * BLK + row;
    t.r[u] = pos < L ? *reinterpret_cast<const uint4 *>(head + (size_t)pos * D + col * 8)
                     : make_uint4(0u, 0u, 0u, 0u);
  }
}

template <int BLK, int STR>
__device__ __forceinline__ void tile_store(uint16_t *lds, int tid, const Tile16 &t)
{
  constexpr int NT = BLK * 2;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int c = tid + NT * u;
    const int row = c >> 3, col = c & 7;
    *reinterpret_cast<uint4 *>(lds + row * STR + col * 8) = t.r[u];
  }
}

}  // namespace

template <int BLK>
__global__ __launch_bounds__(BLK * 2) void fwd_mfma_kernel(const uint16_t *__restrict__ Q,
                                                           const uint16_t *__restrict__ K,
                                                           const uint16_t *__restrict__ V,
                                                           const int *__restrict__ valid_len,
                                                           const int *__restrict__ sel,
                                                           const float *__restrict__ gate_w,
                                                           const float *__restrict__ gate_b,
                                                           uint16_t *__restrict__ O,
                                                           float *__restrict__ o_lt_out,
                                                           float *__restrict__ o_st_out,
                                                           float *__restrict__ lse_lt_out,
                                                           float *__restrict__ lse_st_out, int dense,
                                                           KParams p)
{
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][BLK * KSTR];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][BLK * VSTR];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // readfirstlane tells the compiler the wavefront index is uniform, so every branch that
  // depends on it is a scalar branch: matrix instructions ignore EXEC and must never sit in a
  // region that is merely masked off.
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31;  // query column (and key row of the K operand, d row of the V^T operand)
  const int lh = lane >> 5;  // which half of each 16-wide contraction slab
  const unsigned vid = xcd_remap(blockIdx.x, (unsigned)(p.B * p.H * p.NB));
  const int bh = (int)(vid / p.NB);
  const int I = p.NB - 1 - (int)(vid % p.NB);
  const int h = bh % p.H;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int q0 = I * BLK + 32 * wv;  // first query row of this wavefront
  const int iq = q0 + lq;            // this lane's query row
  const bool q_ok = iq < p.L && iq >= p0;
  const size_t head = (size_t)bh * p.L * D;

  if (min((I + 1) * BLK, p.L) <= p0) {  // no valid query in the block: zero outputs
    if (iq < p.L) {
      const size_t ro = head + (size_t)iq * D + 32 * lh;
#pragma unroll
      for (int c = 0; c < 32; c += 8) *reinterpret_cast<uint4 *>(O + ro + c) = make_uint4(0u, 0u, 0u, 0u);
      if (o_lt_out)
#pragma unroll
        for (int c = 0; c < 32; c += 4) {
          *reinterpret_cast<float4 *>(o_lt_out + ro + c) = make_float4(0.f, 0.f, 0.f, 0.f);
          *reinterpret_cast<float4 *>(o_st_out + ro + c) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      if (lh == 0) {
        if (lse_lt_out) lse_lt_out[(size_t)bh * p.L + iq] = 0.0f;
        if (lse_st_out) lse_st_out[(size_t)bh * p.L + iq] = 0.0f;
      }
    }
    return;
  }

  // Q^T operand: lane (query lq, half lh) holds Q[iq][16*kk + 8*lh .. +7] for the 4 slabs kk.
  bf16x8 qf[4];
  {
    const uint16_t *qrow = Q + head + (size_t)(iq < p.L ? iq : 0) * D;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 v = *reinterpret_cast<const uint4 *>(qrow + 16 * kk + 8 * lh);
      if (iq >= p.L) v = make_uint4(0u, 0u, 0u, 0u);
      qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }

  const int J_first = p0 / BLK;
  const uint16_t *Kh = K + head;
  const uint16_t *Vh = V + head;
  const int *my_sel = dense ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
  int J_lo, n_st, n_all;
  if (dense) {
    J_lo = J_first;
    n_st = 0;
    n_all = I - J_first + 1;
  } else {
    const int lowpos = I * BLK - (p.w - 1);
    J_lo = lowpos <= 0 ? 0 : lowpos / BLK;
    J_lo = max(J_lo, J_first);
    n_st = I - J_lo + 1;
    n_all = n_st + p.k;
  }
  auto tile_of = [&](int t) -> int {  // key block of step t, or -1
    if (dense) return J_first + t;
    if (t < n_st) return J_lo + t;
    const int J = my_sel[t - n_st];
    return (J >= 0 && J < p.NB) ? J : -1;
  };
  auto next_valid = [&](int t) -> int {
    while (t < n_all && tile_of(t) < 0) ++t;
    return t;
  };

  const float c2 = p.scale * kLog2e;
  f32x16 oacc[2];
  float m_run, l_run;
  auto reset = [&]() {
    m_run = kNegInf;
    l_run = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][i] = 0.0f; oacc[1][i] = 0.0f; }
  };
  // normalise the running state into oacc, return lse (natural log)
  auto finish = [&]() -> float {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const bool ok = q_ok && l_tot > 0.0f;
    const float inv = ok ? 1.0f / l_tot : 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][i] *= inv; oacc[1][i] *= inv; }
    return ok ? (m_run + __log2f(l_tot)) * kLn2 : 0.0f;
  };

  // Rows that see only a few keys have large probabilities, and rounding those to bf16 would
  // leave a relative error of 2^-9 in the saved branch outputs, which backward amplifies
  // through D = dO_x.o_x.  Wavefronts that may hold such rows (fewer than kFewKeys keys) feed
  // P to the matrix cores as a two-term bf16 sum (hi + lo); everyone else uses one term.
  constexpr int kFewKeys = 32;
  bool hp_st, hp_lt;
  if (dense) {
    hp_st = false;
    hp_lt = q0 - p0 + 1 < kFewKeys;
  } else {
    hp_st = p.w < kFewKeys || q0 - p0 + 1 < kFewKeys;
    int past = 0;
    for (int e = 0; e < p.k && past < kFewKeys; ++e) {
      const int J = my_sel[e];
      if (J >= 0 && J < I) past += max(0, min((J + 1) * BLK, p.L) - max(J * BLK, p0));
    }
    hp_lt = past < kFewKeys;
  }

  auto compute_tile = [&](int buf, int J, bool windowed) {
    const bool hp = __builtin_amdgcn_readfirstlane((int)(windowed ? hp_st : hp_lt)) != 0;
    const uint16_t *ks = Ks[buf];
    const uint16_t *vs = Vs[buf];
    const bool tile_masked = windowed || J == I || J * BLK < p0;
#pragma unroll
    for (int s = 0; s < BLK / 32; ++s) {
      const int k0 = J * BLK + 32 * s;
      // wave-uniform skips: all keys after all queries, before the window, or all padding
      if (k0 > q0 + 31) continue;
      if (windowed && k0 + 31 < q0 - p.w + 1) continue;
      if (k0 + 31 < p0) continue;
      f32x16 sacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks + (32 * s + lq) * KSTR + 16 * kk + 8 * lh);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc, 0, 0, 0);
      }
      if (tile_masked) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + 8 * (i >> 2) + 4 * lh + (i & 3);
          const bool vis = key <= iq && key >= p0 && (!windowed || iq - key < p.w);
          sacc[i] = vis ? sacc[i] : kNegInf;
        }
      }
      float mx = sacc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx * c2);
      const float m_use = m_new == kNegInf ? 0.0f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      float rs = 0.0f;
      bf16x8 pf[2], pf_lo[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pi = __builtin_amdgcn_exp2f(fmaf(sacc[i], c2, -m_use));
        rs += pi;
        pf[i >> 3][i & 7] = (__bf16)pi;
        sacc[i] = pi;
      }
      if (hp) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          pf_lo[i >> 3][i & 7] = (__bf16)(sacc[i] - (float)pf[i >> 3][i & 7]);
      }
      l_run = l_run * alpha + rs;
      m_run = m_new;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { oacc[0][i] *= alpha; oacc[1][i] *= alpha; }
      }
      // O^T[d][q] += sum_key V^T[d][key] P^T[key][q]
#pragma unroll
      for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const int r16 = lane & 15;
          const int dbase = 32 * mb + 16 * ((lane >> 4) & 1) + 4 * (r16 & 3);
          const int krow = 32 * s + 16 * t + 4 * lh + (r16 >> 2);
          const uint16_t *a0 = vs + krow * VSTR + dbase;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * VSTR));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[t],
                                                             oacc[mb], 0, 0, 0);
          if (hp)
            oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf_lo[t],
                                                               oacc[mb], 0, 0, 0);
        }
      }
    }
  };

  // ---- software pipeline over the tile list ----
  f32x16 ost[2];  // normalised short-term output, parked while the long-term branch runs
  float lse_st = 0.0f;
  bool st_open = !dense;
  reset();
  int t = next_valid(0);
  Tile16 kreg, vreg;
  if (t < n_all) {
    const int J = tile_of(t);
    tile_load<BLK>(Kh, J, p.L, tid, kreg);
    tile_load<BLK>(Vh, J, p.L, tid, vreg);
    tile_store<BLK, KSTR>(Ks[0], tid, kreg);
    tile_store<BLK, VSTR>(Vs[0], tid, vreg);
  }
  __syncthreads();
  int cur = 0;
  while (t < n_all) {
    const int tn = next_valid(t + 1);
    if (tn < n_all) {
      const int Jn = tile_of(tn);
      tile_load<BLK>(Kh, Jn, p.L, tid, kreg);
      tile_load<BLK>(Vh, Jn, p.L, tid, vreg);
    }
    if (st_open && t >= n_st) {  // the window tiles are done: close the short-term branch
      lse_st = finish();
      ost[0] = oacc[0];
      ost[1] = oacc[1];
      reset();
      st_open = false;
    }
    compute_tile(cur, tile_of(t), t < n_st);
    if (tn < n_all) {
      tile_store<BLK, KSTR>(Ks[cur ^ 1], tid, kreg);
      tile_store<BLK, VSTR>(Vs[cur ^ 1], tid, vreg);
    }
    __syncthreads();
    cur ^= 1;
    t = tn;
  }
  if (st_open) {  // a selection list without any usable entry
    lse_st = finish();
    ost[0] = oacc[0];
    ost[1] = oacc[1];
    reset();
  }
  const float lse_lt = finish();

  // ---- epilogue: gate (Eq. 18-19) and stores ----
  if (iq >= p.L) return;
  const size_t rowoff = head + (size_t)iq * D;
  const size_t lrow = (size_t)bh * p.L + iq;
  if (dense) {
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d0 = 32 * mb + 8 * g + 4 * lh;
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(oacc[mb][4 * g]) | ((uint32_t)f32_to_bf16(oacc[mb][4 * g + 1]) << 16);
        pk.y = (uint32_t)f32_to_bf16(oacc[mb][4 * g + 2]) | ((uint32_t)f32_to_bf16(oacc[mb][4 * g + 3]) << 16);
        *reinterpret_cast<uint2 *>(O + rowoff + d0) = pk;
      }
    if (lh == 0 && lse_lt_out) lse_lt_out[lrow] = lse_lt;
    return;
  }
  const float *wl = gate_w + (size_t)h * 2 * D;
  const float *ws = wl + D;
  float z = 0.0f;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int dd = 32 * mb + 8 * (i >> 2) + 4 * lh + (i & 3);
      z = fmaf(wl[dd], oacc[mb][i], z);
      z = fmaf(ws[dd], ost[mb][i], z);
    }
  z += __shfl_xor(z, 32);
  z += gate_b ? gate_b[h] : 0.0f;
  const float alpha = q_ok ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = 32 * mb + 8 * g + 4 * lh;
      float o4[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o4[e] = alpha * oacc[mb][4 * g + e] + (1.0f - alpha) * ost[mb][4 * g + e];
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16(o4[0]) | ((uint32_t)f32_to_bf16(o4[1]) << 16);
      pk.y = (uint32_t)f32_to_bf16(o4[2]) | ((uint32_t)f32_to_bf16(o4[3]) << 16);
      *reinterpret_cast<uint2 *>(O + rowoff + d0) = pk;
      if (o_lt_out) {
        *reinterpret_cast<float4 *>(o_lt_out + rowoff + d0) =
            make_float4(oacc[mb][4 * g], oacc[mb][4 * g + 1], oacc[mb][4 * g + 2], oacc[mb][4 * g + 3]);
        *reinterpret_cast<float4 *>(o_st_out + rowoff + d0) =
            make_float4(ost[mb][4 * g], ost[mb][4 * g + 1], ost[mb][4 * g + 2], ost[mb][4 * g + 3]);
      }
    }
  if (lh == 0) {
    if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
    if (lse_st_out) lse_st_out[lrow] = lse_st;
  }
}

bool fwd_mfma_supported(const KParams &p, int dtype) { return dtype == 1 && p.d == 64 && (p.b == 32 || p.b == 64); }

void launch_fwd_mfma(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  const unsigned grid = (unsigned)(p.B * p.H * p.NB);
  auto u16 = [](const void *x) { return reinterpret_cast<const uint16_t *>(x); };
  if (p.b == 32) {
    hipLaunchKernelGGL((fwd_mfma_kernel<32>), dim3(grid), dim3(64), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.sel, a.gate_w, a.gate_b, (uint16_t *)a.O, (float *)a.o_lt,
                       (float *)a.o_st, a.lse_lt, a.lse_st, a.dense, p);
  } else {
    hipLaunchKernelGGL((fwd_mfma_kernel<64>), dim3(grid), dim3(128), 0, st, u16(a.Q), u16(a.K), u16(a.V),
                       a.valid_len, a.sel, a.gate_w, a.gate_b, (uint16_t *)a.O, (float *)a.o_lt,
                       (float *)a.o_st, a.lse_lt, a.lse_st, a.dense, p);
  }
}

}  // namespace blossom

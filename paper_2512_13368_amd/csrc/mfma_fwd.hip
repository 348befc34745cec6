// Fused forward on the matrix cores for bf16, d = 64, block size 32 or 64 (Eq. 1 under the two
// branch masks, Eq. 16-19), plus the same-style dense causal comparison.
//
// Work split: one workgroup per (row, head, query block); one wavefront per 32 query rows.
// K/V tiles of the short-term window and of the selected blocks are gathered by the selection
// list with direct global->LDS loads (16 bytes per lane, whole 128-byte rows per 8 lanes),
// double buffered, XOR-swizzled so that the operand reads below are bank-conflict free, and
// shared by the workgroup's wavefronts.
//
// Per 32-key unit a wavefront computes S^T = K Q^T with four v_mfma_f32_32x32x16_bf16 (keys
// are the M dimension, so every lane owns ONE query column and 16 of its logits: row maximum
// and row sum are in-lane reductions plus one exchange with lane^32), applies the online
// softmax in fp32, and feeds P^T straight from the accumulator registers (converted to bf16)
// as the B operand of O^T += V^T P^T (four more MFMAs).  The key order inside a contraction
// slab is whatever the accumulator layout dictates; V^T is read from LDS with the transposing
// ds_read_b64_tr_b16 in exactly that order, so P never moves between lanes.
//
// Pipeline: the logits of tile t+1 are issued to the matrix cores in the same straight-line
// region as the exponentials of tile t and its P V products, so MFMA and VALU work of one
// wavefront can overlap; K therefore runs one tile ahead of V in LDS.
//
// Softmax bookkeeping: Q is pre-multiplied by scale*log2(e) (rounded to bf16 once), and the
// logits accumulator of a tile starts at minus the row's current reference m_ref instead of
// zero, so the MFMA result is directly the exponent s*c - m_ref and each probability costs one
// v_exp_f32.  m_ref is only moved when a row's tile maximum exceeds 2^8 above it (then the
// tile's exponents, the running sum and the output accumulators are shifted), or on the first
// visible key of a branch; probabilities therefore stay below 2^8, far inside bf16 range.
#include "common.h"
#include "launch.h"

namespace blossom {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kRaise = 8.0f;  // log2 units by which the maximum must grow before it is raised
constexpr int kMaxTiles = 96;   // window blocks + selected blocks one query block may walk (host-checked)
constexpr int kFewKeys = 32;    // rows seeing fewer keys than this get two-term bf16 probabilities

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// Maps the hardware workgroup id (dealt round-robin over the 8 XCDs) to a virtual id such that
// each XCD works through a contiguous range: all query blocks of a head then share one L2.
__device__ __forceinline__ unsigned xcd_remap(unsigned pid, unsigned total)
{
  constexpr unsigned X = 8;
  const unsigned per = (total + X - 1) / X;  // ids of a "tall" XCD
  const unsigned tall = total % X ? total % X : X;
  const unsigned xcd = pid % X, local = pid / X;
  return xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
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
  constexpr int UNITS = BLK / 32;  // 32-key units per tile
  constexpr int TILE = BLK * D;    // bf16 elements of one staged tile (rows of 128 bytes, swizzled)
  // Four separate arrays (not one indexed by parity): the compiler can then prove that a
  // prefetch in flight into one buffer does not alias the operand reads of another, and does
  // not wait for the prefetch before those reads.
  __shared__ __attribute__((aligned(1024))) uint16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs1[TILE];
  __shared__ int tiles[kMaxTiles];  // key blocks in processing order: window blocks, then selected blocks
  __shared__ float gate_s[2 * D];   // this head's gate weights, fetched at the start, used at the very end

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
  const int q0 = I * BLK + 32 * wv;  // first query row of this wavefront
  const int iq = q0 + lq;            // this lane's query row
  const size_t head = (size_t)bh * p.L * D;

  // ---- everything the prologue needs from memory is requested before anything is waited for ----
  const int n_raw = valid_len[bh / p.H];
  uint4 qraw[4];
  {
    const uint16_t *qrow = Q + head + (size_t)min(iq, p.L - 1) * D;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qraw[kk] = *reinterpret_cast<const uint4 *>(qrow + 16 * kk + 8 * lh);
  }
  const int *my_sel = dense ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
  const int sel0 = (!dense && lane < p.k) ? my_sel[lane] : -1;  // first 64 entries of the selection row
  constexpr int GATE_PER = 2 * D / (2 * BLK);  // gate weights fetched per thread
  float gate_mine[GATE_PER];
#pragma unroll
  for (int c = 0; c < GATE_PER; ++c) gate_mine[c] = dense ? 0.0f : gate_w[(size_t)h * 2 * D + c * 2 * BLK + tid];

  const int n = clamp_len(n_raw, p.L);
  const int p0 = p.L - n;
  const bool q_ok = iq < p.L && iq >= p0;

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

  // window blocks J_lo..I come first in the walk; they depend on the valid length only
  const int J_first = p0 / BLK;
  int J_lo, n_st;
  if (dense) {
    J_lo = J_first;
    n_st = 0;
  } else {
    const int lowpos = I * BLK - (p.w - 1);
    J_lo = lowpos <= 0 ? 0 : lowpos / BLK;
    J_lo = max(J_lo, J_first);
    n_st = I - J_lo + 1;
  }

  // ---- staging: each wavefront moves 4 x 1 KB of K and of V per tile ----
  // LDS position of 16-byte chunk c of row r:  r*128 + ((c ^ swz(r)) * 16),
  //   swzK(r) = r & 7 (8 rows x one chunk column = 8 distinct positions for the row-per-lane reads)
  //   swzV(r) = 2*(r & 3) (4 rows x two chunk columns = 8 distinct positions for the transposing reads)
  const uint16_t *Kh = K + head;
  const uint16_t *Vh = V + head;
  const int ld_row = 32 * wv + (lane >> 3);  // + 8*u
  const int ld_ck = ((lane & 7) ^ (lane >> 3)) * 8;
  const int ld_cv = ((lane & 7) ^ (2 * ((lane >> 3) & 3))) * 8;
  const uint16_t *k_lane = Kh + ld_row * D + ld_ck;  // this lane's chunk inside block 0
  const uint16_t *v_lane = Vh + ld_row * D + ld_cv;
  const bool ragged = p.L % BLK != 0;
  auto stage = [&](const uint16_t *src_lane, uint16_t *dst_tile, int J) {
    if (!ragged || J != p.NB - 1) {
      const uint16_t *src = src_lane + (size_t)J * TILE;  // lane pointer + uniform tile offset
#pragma unroll
      for (int u = 0; u < 4; ++u)
        __builtin_amdgcn_global_load_lds((glb_void *)(src + 8 * u * D),
                                         (lds_void *)(dst_tile + (32 * wv + 8 * u) * D), 16, 0, 0);
    } else {  // last, partial block: rows past the end are clamped (they are causally masked anyway)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int over = max(0, J * BLK + ld_row + 8 * u - (p.L - 1));
        const uint16_t *src = src_lane + (size_t)J * TILE + (8 * u - over) * D;
        __builtin_amdgcn_global_load_lds((glb_void *)src, (lds_void *)(dst_tile + (32 * wv + 8 * u) * D), 16, 0, 0);
      }
    }
  };

  // the first tiles are on their way while the rest of the prologue runs
  const int first_J = dense ? J_first : J_lo;
  const bool second_known = dense ? (I > J_first) : (n_st > 1);  // tile 1 is first_J + 1
  stage(k_lane, Ks0, first_J);
  stage(v_lane, Vs0, first_J);
  if (second_known) stage(k_lane, Ks1, first_J + 1);

  // Q^T operand: lane (query lq, half lh) holds c*Q[iq][16*kk + 8*lh .. +7] for the 4 slabs kk,
  // c = scale*log2(e), rounded to bf16: the matrix cores then produce base-2 exponents directly.
  const float c2 = p.scale * kLog2e;
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const uint32_t w[4] = {qraw[kk].x, qraw[kk].y, qraw[kk].z, qraw[kk].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qf[kk][2 * e] = (__bf16)(__uint_as_float(w[e] << 16) * c2);
      qf[kk][2 * e + 1] = (__bf16)(__uint_as_float(w[e] & 0xFFFF0000u) * c2);
    }
  }
  if (!dense)
#pragma unroll
    for (int c = 0; c < GATE_PER; ++c) gate_s[c * 2 * BLK + tid] = gate_mine[c];

  // ---- tile list: window blocks J_lo..I, then the selection list up to its first -1 ----
  // Every wavefront reads the whole selection row with one vector load per 64 entries and
  // derives the counts from ballots (no chain of dependent scalar loads); the list itself is
  // parked in LDS so that walking it never waits on the vector-memory counter, which also
  // tracks the tile prefetches in flight.
  int n_all;
  bool lt_few = true;  // the selected past blocks hold fewer than kFewKeys valid keys
  if (dense) {
    n_all = I - J_first + 1;
  } else {
    if (wv == 0)
      for (int t = lane; t < n_st; t += 64) tiles[t] = J_lo + t;
    int n_lt = 0;
    bool open = true;
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      const int e = e0 + lane;
      const int J = e0 == 0 ? sel0 : (e < p.k ? my_sel[e] : -1);
      const bool ok = J >= 0 && J < p.NB;
      const unsigned long long okm = __ballot(ok);
      const int lead = okm == ~0ull ? 64 : __builtin_ctzll(~okm);  // entries before the first -1
      if (open) {
        const bool mine = lane < lead;
        if (wv == 0 && mine) tiles[n_st + e] = J;
        // a full earlier block already brings a whole block of keys; only a partial first block may not
        const int vcount = min((J + 1) * BLK, p.L) - max(J * BLK, p0);
        if (__ballot(mine && J < I && vcount >= kFewKeys) != 0ull) lt_few = false;
        n_lt += lead;
        open = lead == 64;
      }
    }
    n_all = n_st + n_lt;
  }
  __syncthreads();
  auto tile_of = [&](int t) -> int {
    if (dense) return J_first + t;
    return __builtin_amdgcn_readfirstlane(tiles[t]);
  };
  if (!second_known && n_all > 1) stage(k_lane, Ks1, tile_of(1));

  // ---- per-lane LDS read offsets (elements) ----
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = lq * D + (((2 * kk + lh) ^ (lq & 7)) * 8);
  const int r16 = lane & 15;
  int voff[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
    voff[mb] = (4 * lh + (r16 >> 2)) * D +
               (((4 * mb + 2 * ((lane >> 4) & 1) + ((r16 & 3) >> 1)) ^ (2 * (r16 >> 2))) * 8) + 4 * (r16 & 1);

  // Per-row softmax state.  m_ref: reference exponent (log2 units) the accumulators are relative
  // to; fresh: nothing accumulated yet in this branch; l_run: this lane's part of the row sum.
  f32x16 oacc[2];
  float m_ref = 0.0f, l_run;
  bool fresh;
  auto reset = [&]() {
    fresh = true;
    l_run = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][i] = 0.0f; oacc[1][i] = 0.0f; }
  };
  auto finish = [&]() -> float {  // normalise the running state into oacc, return lse (natural log)
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const bool ok = q_ok && l_tot > 0.0f;
    const float inv = ok ? 1.0f / l_tot : 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][i] *= inv; oacc[1][i] *= inv; }
    return ok ? (m_ref + __log2f(l_tot)) * kLn2 : 0.0f;
  };
  // exponents of one tile: sacc = c*K Q^T - m_ref
  auto qk = [&](const uint16_t *ks, f32x16 (&sacc)[UNITS]) {
    const float init = -m_ref;
#pragma unroll
    for (int s = 0; s < UNITS; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[s][i] = init;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int s = 0; s < UNITS; ++s) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks + 32 * s * D + koff[kk]);
        sacc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[s], 0, 0, 0);
      }
  };

  // Rows that see only a few keys have large probabilities, and rounding those to bf16 would
  // leave a relative error of 2^-9 in the saved branch outputs, which backward amplifies
  // through D = dO_x.o_x.  Wavefronts that may hold such rows (fewer than kFewKeys keys) feed
  // P to the matrix cores as a two-term bf16 sum (hi + lo); everyone else uses one term.
  bool hp_st, hp_lt;
  if (dense) {
    hp_st = false;
    hp_lt = q0 - p0 + 1 < kFewKeys;
  } else {
    hp_st = p.w < kFewKeys || q0 - p0 + 1 < kFewKeys;
    hp_lt = lt_few;
  }

  // ---- per-tile pieces ----
  // prep: mask the exponents of tile J and move the row reference if needed (see file header).
  auto prep = [&](int J, bool windowed, f32x16 (&sacc)[UNITS]) {
    if (windowed || J == I || J * BLK < p0) {
      // visible <=> lo <= key <= iq with lo = max(p0, iq - w + 1); per lane this is one range
      // test on the element's compile-time key offset
      const int lo = windowed ? max(p0, iq - p.w + 1) : p0;
      const int base = J * BLK + 4 * lh;
      const unsigned span = (unsigned)(iq - lo);  // wraps to huge when iq < lo: handled by q-validity below
      const bool any = iq >= lo;
#pragma unroll
      for (int s = 0; s < UNITS; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = base + 32 * s + 8 * (i >> 2) + (i & 3);
          const bool vis = any & ((unsigned)(key - lo) <= span);
          sacc[s][i] = vis ? sacc[s][i] : kNegInf;
        }
    }
    float m4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) m4[c] = sacc[0][c];
#pragma unroll
    for (int s = 0; s < UNITS; ++s)
#pragma unroll
      for (int i = (s == 0 ? 4 : 0); i < 16; ++i) m4[i & 3] = fmaxf(m4[i & 3], sacc[s][i]);
    float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    {  // other half of the row lives in lane^32
      const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    // move the reference: first visible key of the branch, or the tile maximum ran away upwards
    const bool upd = fresh ? mx != kNegInf : mx > kRaise;
    if (__any(upd)) {
      const float dlt = upd ? mx : 0.0f;
      const float alpha = (upd && !fresh) ? __builtin_amdgcn_exp2f(-dlt) : 1.0f;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < 16; ++i) { oacc[0][i] *= alpha; oacc[1][i] *= alpha; }
#pragma unroll
      for (int s = 0; s < UNITS; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[s][i] -= dlt;
      m_ref += dlt;
      fresh = fresh && !upd;
    }
  };

  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  // exponentials of one 32-key unit: sacc <- p (fp32), pf <- bf16(p), l_run += sum of bf16(p)
  auto expo = [&](f32x16 &sacc, bf16x8 (&pf)[2]) {
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float pa = __builtin_amdgcn_exp2f(sacc[i]);
      const float pb = __builtin_amdgcn_exp2f(sacc[i + 1]);
      sacc[i] = pa;
      sacc[i + 1] = pb;
      const bf16x2 pk = {(__bf16)pa, (__bf16)pb};
      pf[i >> 3][i & 7] = pk[0];
      pf[i >> 3][(i & 7) + 1] = pk[1];
      l_run = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run, false);  // sums what the MFMA will see
    }
  };
  // V^T operands of one unit: [t][mb], keys in accumulator order
  auto load_v = [&](const uint16_t *vs, int s, bf16x8 (&vf)[2][2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const uint16_t *a0 = vs + (32 * s + 16 * t) * D + voff[mb];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * D));
        vf[t][mb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
  };
  auto pv = [&](const bf16x8 (&vf)[2][2], const bf16x8 (&pf)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][mb], pf[t], oacc[mb], 0, 0, 0);
  };

  // One tile: logits of the next tile (K from ks_next), exponentials of this one and P V.
  auto tile_body = [&](const uint16_t *vs, const uint16_t *ks_next, bool windowed,
                       f32x16 (&sacc)[UNITS], f32x16 (&snext)[UNITS]) {
    const bool hp = __builtin_amdgcn_readfirstlane((int)(windowed ? hp_st : hp_lt)) != 0;
    bf16x8 kf[UNITS][4];
#pragma unroll
    for (int s = 0; s < UNITS; ++s)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kf[s][kk] = *reinterpret_cast<const bf16x8 *>(ks_next + 32 * s * D + koff[kk]);
    bf16x8 vf[2][2];
    load_v(vs, 0, vf);
    const float init = -m_ref;
#pragma unroll
    for (int s = 0; s < UNITS; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) snext[s][i] = init;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int s = 0; s < UNITS; ++s)
        snext[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][kk], qf[kk], snext[s], 0, 0, 0);
    bf16x8 pf[UNITS][2];
#pragma unroll
    for (int s = 0; s < UNITS; ++s) {
      expo(sacc[s], pf[s]);
      pv(vf, pf[s]);
      if (s + 1 < UNITS) load_v(vs, s + 1, vf);
    }
    if (hp) {  // second bf16 term of P
#pragma unroll
      for (int s = 0; s < UNITS; ++s) {
        bf16x8 pl[2];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const bf16x2 pk = {(__bf16)(sacc[s][i] - (float)pf[s][i >> 3][i & 7]),
                             (__bf16)(sacc[s][i + 1] - (float)pf[s][i >> 3][(i & 7) + 1])};
          pl[i >> 3][i & 7] = pk[0];
          pl[i >> 3][(i & 7) + 1] = pk[1];
          l_run = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run, false);
        }
        load_v(vs, s, vf);
        pv(vf, pl);
      }
    }
  };

  // ---- pipeline over the tile list: K runs one tile ahead of V ----
  f32x16 ost[2];  // normalised short-term output, parked while the long-term branch runs
  float lse_st = 0.0f;
  bool st_open = !dense;
  reset();
  f32x16 sA[UNITS], sB[UNITS];
  __syncthreads();
  qk(Ks0, sA);
  __syncthreads();  // Ks0 may be overwritten from here on
  auto close_st = [&]() {
    lse_st = finish();
    ost[0] = oacc[0];
    ost[1] = oacc[1];
    reset();
    st_open = false;
  };
  if (st_open && n_st == 0) close_st();
  prep(tile_of(0), 0 < n_st, sA);

  // step t: prefetch K(t+2) and V(t+1); exponentials and P V of tile t; logits, mask and
  // maximum of tile t+1 (the latter overlap the last P V products)
  auto step = [&](int t, uint16_t *k_fill, uint16_t *v_fill, const uint16_t *v_cur, const uint16_t *k_next,
                  f32x16 (&scur)[UNITS], f32x16 (&snext)[UNITS]) {
    if (t + 2 < n_all) stage(k_lane, k_fill, tile_of(t + 2));
    if (t + 1 < n_all) stage(v_lane, v_fill, tile_of(t + 1));
    tile_body(v_cur, k_next, t < n_st, scur, snext);
    if (st_open && t + 1 >= n_st) close_st();  // the window tiles are done: close the short-term branch
    if (t + 1 < n_all) prep(tile_of(t + 1), t + 1 < n_st, snext);
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Ks0, Vs1, Vs0, Ks1, sA, sB);
    if (t + 1 < n_all) step(t + 1, Ks1, Vs0, Vs1, Ks0, sB, sA);
  }
  if (st_open) {  // no usable selection entry at all
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
  const float *wl = gate_s;
  const float *ws = gate_s + D;
  float z = 0.0f;
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = 32 * mb + 8 * g + 4 * lh;
      const float4 a = *reinterpret_cast<const float4 *>(wl + d0);
      const float4 b = *reinterpret_cast<const float4 *>(ws + d0);
      z = fmaf(a.x, oacc[mb][4 * g], z);
      z = fmaf(a.y, oacc[mb][4 * g + 1], z);
      z = fmaf(a.z, oacc[mb][4 * g + 2], z);
      z = fmaf(a.w, oacc[mb][4 * g + 3], z);
      z = fmaf(b.x, ost[mb][4 * g], z);
      z = fmaf(b.y, ost[mb][4 * g + 1], z);
      z = fmaf(b.z, ost[mb][4 * g + 2], z);
      z = fmaf(b.w, ost[mb][4 * g + 3], z);
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

bool fwd_mfma_supported(const KParams &p, int dtype)
{
  if (dtype != 1 || p.d != 64 || (p.b != 32 && p.b != 64)) return false;
  // window blocks (at most (w-1)/b + 2) plus selected blocks must fit the in-LDS tile list
  return (long)(p.w - 1) / p.b + 2 + p.k <= kMaxTiles;
}

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

// Fused forward on the matrix cores for bf16, d = 64, block size 64 (Eq. 1 under the two branch
// masks, Eq. 16-19), plus the same-style dense causal comparison: the four-wavefront form.
//
// One workgroup per (row, head, query block), four wavefronts.  Wavefront (qg, kh) works on the 32
// query rows of group qg and on the 32 key rows of half kh of every K/V tile, so a wavefront carries
// half of the accumulators of a wavefront that holds all 64 query rows: 3 wavefronts per SIMD fit
// the register file (12 per CU instead of 8), and the phases that use no matrix pipe (prologue,
// branch merges, epilogue, memory waits) of one workgroup are covered by more resident ones.
// A tile is staged cooperatively (each wavefront moves 16 of its 64 rows of K and of V with direct
// global->LDS loads) and read by all four, so the tile loop has one workgroup barrier per tile;
// tiles are requested two steps ahead into three buffer pairs.
//
// Per tile a wavefront computes S^T = K Q^T with four v_mfma_f32_32x32x16_bf16 (keys are the M
// dimension: a lane owns one query column and 16 of its logits), the first of which takes minus the
// row's softmax reference as its C operand (a 16-register block), so the result is directly the
// base-2 exponent; then the online softmax in fp32 and O^T += V^T P^T with P^T straight from the
// accumulator registers and V^T through the transposing LDS read.  Reference bookkeeping, masks,
// two-term probabilities for rows with few keys and the walk are those of the two-wavefront kernel
// in mfma_fwd.hip, which keeps serving block size 32.
//
// At the end of a branch the two wavefronts of a query group hold partial results over disjoint key
// halves; they are merged through the staging rows that were just consumed, and afterwards
// wavefront (qg, kh) owns channels 32*kh .. 32*kh+31 of the finished rows 32*qg .. 32*qg+31.
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

using namespace mfma;

namespace {

constexpr float kRaise4 = 8.0f;        // log2 units by which the maximum must grow before the reference is raised
constexpr int kFewKeys4 = 32;          // rows seeing fewer keys than this get two-term bf16 probabilities
constexpr float kSumLimit4 = 4096.0f;  // a lane's 16 probabilities of a tile may sum to this (16 * 2^kRaise4)
constexpr int BLK4 = 64;

constexpr int vmcnt_imm4(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

}  // namespace

template <bool EQ15, bool SUB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void fwd_mfma4_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int *__restrict__ valid_len, const int *__restrict__ sel, const float *__restrict__ gate_w,
    const float *__restrict__ gate_b, uint16_t *__restrict__ O, float *__restrict__ o_lt_out,
    float *__restrict__ o_st_out, float *__restrict__ lse_lt_out, float *__restrict__ lse_st_out, int dense,
    KParams p)
{
  constexpr int BLK = BLK4;
  constexpr int TILE = BLK * D;  // bf16 elements of one staged tile (rows of 128 bytes, swizzled)
  constexpr int HALF = 32 * D;   // elements of the 32 key rows one wavefront reads
  __shared__ __attribute__((aligned(1024))) uint16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks2[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs2[TILE];
  __shared__ float gate_s[2 * D];  // this head's gate weights
  __shared__ float xch_s[4][3][32];  // per wavefront: reference, row sum (branch merge), gate partial

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // (uniform through readfirstlane: every branch on them is scalar, as matrix instructions need)
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qg = wv & 1;   // query group: rows 32*qg .. 32*qg+31 of the block
  const int kh = wv >> 1;  // key half: rows 32*kh .. 32*kh+31 of every tile; after a merge: channels 32*kh ..
  const int lq = lane & 31;
  const int lh = lane >> 5;
  const unsigned vid = xcd_remap(blockIdx.x, (unsigned)(p.B * p.H * p.nq));
  const int bh = (int)(vid / p.nq);
  const int I = p.NB - 1 - (int)(vid % p.nq);
  const int h = bh % p.H;
  const size_t head = (size_t)bh * p.L * D;
  const int qbase = I * BLK + 32 * qg;
  const int iq = qbase + lq;

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
  const float gate_mine = (dense || tid >= 2 * D) ? 0.0f : gate_w[(size_t)h * 2 * D + tid];

  const int n = clamp_len(n_raw, p.L);
  const int p0 = p.L - n;
  const bool q_ok = iq < p.L && iq >= p0;

  if (min((I + 1) * BLK, p.L) <= p0) {  // no valid query in the block: zero outputs (16 rows per wavefront)
    const int zr = I * BLK + 16 * wv;
    zero_rows(O + head, zr, 16, p.L, lane);
    if (o_lt_out) {
      zero_rows(o_lt_out + head, zr, 16, p.L, lane);
      zero_rows(o_st_out + head, zr, 16, p.L, lane);
    }
    if (iq < p.L && lh == 0 && kh == 0) {
      if (lse_lt_out) lse_lt_out[(size_t)bh * p.L + iq] = 0.0f;
      if (lse_st_out) lse_st_out[(size_t)bh * p.L + iq] = 0.0f;
    }
    return;
  }

  // window blocks J_lo..I come first in the walk; with the full short-term mask (Eq. 15) the blocks
  // I - 2^r below the window range follow (see mfma_fwd.hip for the variants EQ15 and SUB)
  const int J_first = p0 / BLK;
  constexpr bool sub = EQ15 && SUB;
  const int sub_sh = sub ? __builtin_ctz((unsigned)p.sblk) : 0;
  int J_lo, n_win, n_st, r0 = 0;
  if (dense) {
    J_lo = J_first;
    n_win = 0;
    n_st = 0;
  } else {
    const int lowpos = I * BLK - (p.w - 1);
    J_lo = lowpos <= 0 ? 0 : lowpos / BLK;
    if (sub) J_lo = min(J_lo, I - 1);
    J_lo = max(J_lo, J_first);
    n_win = I - J_lo + 1;
    n_st = n_win;
    if (EQ15 && I > J_first) {
      const int d_win = I - J_lo;
      r0 = d_win == 0 ? 0 : 32 - __builtin_clz((unsigned)d_win);
      const int r_max = 31 - __builtin_clz((unsigned)(I - J_first));
      n_st += max(0, r_max - r0 + 1);
    }
  }

  // ---- staging: each wavefront moves 16 rows (2 x 1 KB) of K and of V per tile ----
  // LDS position of 16-byte chunk c of row r: r*128 + ((c ^ swz(r)) * 16), swzK(r) = (r >> 1) & 7 for
  // the row-per-lane 16-byte reads, swzV(r) = 2*(r & 3) for the transposing reads (both measured
  // conflict free).  A tile's rows are contiguous in memory and the LDS copy keeps the 128-byte row
  // pitch: one uniform base + one per-lane byte offset + an immediate address both 8-row slices.
  const char *Kh = reinterpret_cast<const char *>(K + head);
  const char *Vh = reinterpret_cast<const char *>(V + head);
  const int ld_row = 16 * wv + (lane >> 3);  // + 8 for the second slice
  const unsigned k_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (lane >> 4)) * 8) * 2u;            // bytes
  const unsigned v_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (2 * ((lane >> 3) & 3))) * 8) * 2u;  // bytes
  // (offsets inside a head stay below 2^31 bytes: one uniform 64-bit base per tensor, 32-bit lane offsets)
  const int J_rag = p.L % BLK != 0 ? p.NB - 1 : -2;  // the one block whose rows run past the end, if any
  auto stage = [&](const char *src_head, unsigned lane_off, unsigned odd_xor, uint16_t *dst_tile, int J) __attribute__((always_inline)) {
    const unsigned joff = (unsigned)max(J, 0) * (unsigned)(TILE * 2);  // uniform (block -1: a skipped list entry, all masked)
    lds_void *dst = (lds_void *)(dst_tile + 16 * wv * D);
    if (J != J_rag) {
      __builtin_amdgcn_global_load_lds((glb_void *)(src_head + (joff + lane_off)), dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src_head + (joff + (lane_off ^ odd_xor))), dst, 16, 1024, 0);
    } else {  // last, partial block: rows past the end are clamped (they are causally masked anyway)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int over = max(0, J * BLK + ld_row + 8 * u - (p.L - 1));
        const unsigned off = joff + ((u & 1) ? lane_off ^ odd_xor : lane_off) + (unsigned)((8 * u - over) * D * 2);
        __builtin_amdgcn_global_load_lds((glb_void *)(src_head + off), (lds_void *)(dst_tile + (16 * wv + 8 * u) * D), 16, 0, 0);
      }
    }
  };

  // the first tile is on its way while the rest of the prologue runs
  const int first_J = dense ? J_first : J_lo;
  stage(Kh, k_lane, 64u, Ks0, first_J);
  stage(Vh, v_lane, 0u, Vs0, first_J);

  // Q^T operand: lane (query lq, half lh) holds c*Q[iq][16*kk + 8*lh .. +7], c = scale*log2(e), in bf16
  const float c2 = p.scale * kLog2e;
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const uint32_t w[4] = {qraw[kk].x, qraw[kk].y, qraw[kk].z, qraw[kk].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qf[kk][2 * e] = (__bf16)(bf_lo(w[e]) * c2);
      qf[kk][2 * e + 1] = (__bf16)(bf_hi(w[e]) * c2);
    }
  }
  if (!dense && tid < 2 * D) gate_s[tid] = gate_mine;

  // ---- tile list: window blocks J_lo..I, then the selection list up to its last valid entry ----
  int n_all;
  bool lt_few = true;  // the selected past blocks hold fewer than kFewKeys4 valid keys
  if (dense) {
    n_all = I - J_first + 1;
  } else {
    int n_lt = 0;
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      const int e = e0 + lane;
      const int J = e0 == 0 ? sel0 : (e < p.k ? my_sel[e] : -1);
      const bool ok = J >= 0 && J < p.NB;
      const unsigned long long okm = __ballot(ok);
      if (okm != 0ull) n_lt = e0 + 64 - __builtin_clzll(okm);
      const int vcount = min((J + 1) * BLK, p.L) - max(J * BLK, p0);
      if (__ballot(ok && J < I && vcount >= kFewKeys4) != 0ull) lt_few = false;
    }
    n_all = n_st + n_lt;
  }
  // The tile list, 64 entries at a time in one register (lane l: entry 64*c + l): window blocks by
  // arithmetic, then the selection row; entries outside [0, NB) and entries past the end are -1 (a tile
  // whose keys are all masked).  A step takes its block id with one v_readlane.
  auto list_chunk = [&](int c) __attribute__((always_inline)) -> int {
    const int t = 64 * c + lane;
    int J;
    if (dense) {
      J = J_first + t;
    } else if (t < n_st) {
      J = (!EQ15 || t < n_win) ? J_lo + t : I - (1 << min(r0 + t - n_win, 30));
    } else {
      const int e = t - n_st;
      J = e < p.k ? (e < 64 && n_st == 0 ? sel0 : my_sel[e]) : -1;
      J = (unsigned)J < (unsigned)p.NB ? J : -1;
    }
    return t < n_all ? J : -1;
  };
  int tl = list_chunk(0);
  auto list_at = [&](int t) __attribute__((always_inline)) -> int {
    return __builtin_amdgcn_readlane(tl, t & 63);
  };

  // ---- per-lane LDS read offsets (elements) inside the 32 key rows of half kh ----
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = kh * HALF + lq * D + (((2 * kk + lh) ^ ((lq >> 1) & 7)) * 8);
  const int r16 = lane & 15;
  int voff[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
    voff[mb] = kh * HALF + (4 * lh + (r16 >> 2)) * D +
               (((4 * mb + 2 * ((lane >> 4) & 1) + ((r16 & 3) >> 1)) ^ (2 * (r16 >> 2))) * 8) + 4 * (r16 & 1);

  // Softmax state.  m_ref: reference exponent (log2 units); fresh: no visible key met yet in this
  // branch; l_run: this lane's part of the row sum.  sinit holds -m_ref in all 16 slots: the first
  // matrix instruction of a tile's logits takes it as its C operand.
  f32x16 oacc[2], sinit;
  float m_ref, l_run;
  bool fresh;
  auto set_ref = [&](float m) __attribute__((always_inline)) {
    m_ref = m;
#pragma unroll
    for (int i = 0; i < 16; ++i) sinit[i] = -m;
    asm volatile("" : "+v"(sinit));  // a register block, not one value copied at each use
  };
  set_ref(0.0f);
  auto reset = [&]() __attribute__((always_inline)) {
    fresh = q_ok;
    l_run = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][i] = 0.0f; oacc[1][i] = 0.0f; }
  };

  const int J_whole = (p0 + BLK - 1) / BLK;  // first block without padding
  int hp_st, hp_lt;  // uniform: blocks whose rows may see fewer than kFewKeys4 keys feed P as hi + lo
  if (dense) {
    hp_st = 0;
    hp_lt = I * BLK - p0 + 1 < kFewKeys4;
  } else {
    hp_st = p.w < kFewKeys4 || I * BLK - p0 + 1 < kFewKeys4;
    hp_lt = __builtin_amdgcn_readfirstlane((int)lt_few);
  }

  // visible <=> lo <= key <= iq with lo = max(p0, iq - w + 1); per lane one range test on the element's
  // compile-time key offset
  auto mask = [&](int J, bool windowed, f32x16 &s) __attribute__((always_inline)) {
    int ql;  // (rebuilt from the lane id inside a volatile asm so that nothing below is hoisted out of the walk)
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ql));
    const int q = qbase + (ql & 31);
    const int lh_ = ql >> 5;
    asm volatile("" : "+s"(J));
    int wlo = q - p.w + 1;
    if (EQ15 && q >= p.last_lo) wlo = min(wlo, p.last_lo);  // third case of Eq. 15
    const int lo = windowed ? max(p0, wlo) : p0;
    const int base = J * BLK + 32 * kh + 4 * lh_;
    const unsigned span = (unsigned)(q - lo);
    const bool any = q >= lo;
    if (EQ15 && sub && windowed && J < J_lo && J * BLK >= p0) {
      const int qo = q & (BLK - 1);
      const int kb = 32 * kh + 4 * lh_;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int ko = kb + 8 * (i >> 2) + (i & 3);
        s[i] = (((qo ^ ko) >> sub_sh) == 0 && q >= p0) ? s[i] : kNegInf;
      }
      return;
    }
    if (EQ15 && sub && windowed) {
      const unsigned cspan = (unsigned)(q - p0);
      const bool cany = q >= p0;
      const int qmb = q >> sub_sh;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = base + 8 * (i >> 2) + (i & 3);
        const int x = qmb - (key >> sub_sh);
        const bool far = cany & ((unsigned)(key - p0) <= cspan) & ((x > 0 && (x & (x - 1)) == 0) | (key >= p.last_lo));
        const bool vis = (any & ((unsigned)(key - lo) <= span)) | far;
        s[i] = vis ? s[i] : kNegInf;
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = base + 8 * (i >> 2) + (i & 3);
      const bool vis = any & ((unsigned)(key - lo) <= span);
      s[i] = vis ? s[i] : kNegInf;
    }
  };
  auto row_max = [&](const f32x16 &s) __attribute__((always_inline)) -> float {
    float m4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) m4[c] = s[c];
#pragma unroll
    for (int i = 4; i < 16; ++i) m4[i & 3] = fmaxf(m4[i & 3], s[i]);
    float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  };
  // slow path of the reference bookkeeping (first visible key of a row, or a maximum that ran away)
  auto move_ref = [&](f32x16 &s) __attribute__((always_inline)) {
    const float mx = row_max(s);
    const bool upd = fresh ? mx != kNegInf : mx > kRaise4;
    const float dlt = upd ? mx : 0.0f;
    if (__any(upd && !fresh)) {  // (a row that has met no key yet has nothing to rescale)
      const float alpha = (upd && !fresh) ? __builtin_amdgcn_exp2f(-dlt) : 1.0f;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < 16; ++i) { oacc[0][i] *= alpha; oacc[1][i] *= alpha; }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] -= dlt;
    set_ref(m_ref + dlt);
    fresh = fresh && !upd;
  };
  auto expo = [&](const f32x16 &s, bf16x8 (&pf)[2]) __attribute__((always_inline)) -> float {
    float sum_a = 0.0f, sum_b = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float pa = __builtin_amdgcn_exp2f(s[i]);
      const float pb = __builtin_amdgcn_exp2f(s[i + 1]);
      pf[i >> 3][i & 7] = (__bf16)pa;
      pf[i >> 3][(i & 7) + 1] = (__bf16)pb;
      sum_a += pa;
      sum_b += pb;
    }
    return sum_a + sum_b;
  };
  auto expo_lo = [&](const f32x16 &s, const bf16x8 (&pf)[2], bf16x8 (&pl)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      pl[i >> 3][i & 7] = (__bf16)(__builtin_amdgcn_exp2f(s[i]) - (float)pf[i >> 3][i & 7]);
  };
  auto pv = [&](const bf16x8 (&vf)[2][2], const bf16x8 (&pf)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][mb], pf[t], oacc[mb], 0, 0, 0);
  };

  // One tile: this wavefront's 32 keys of block J against its 32 queries.
  auto tile = [&](const uint16_t *ks, const uint16_t *vs, int J, bool short_term) __attribute__((always_inline)) {
    const bool hp = (short_term ? hp_st : hp_lt) != 0;
    const bool windowed = short_term && !(EQ15 && !sub && is_pow2(I - J));
    asm volatile("" : "+v"(koff[0]), "+v"(koff[1]), "+v"(koff[2]), "+v"(koff[3]), "+v"(voff[0]), "+v"(voff[1]));
    // long-term tiles of whole earlier blocks (the usual case) need neither a mask nor any other test
    bool full = !short_term && (unsigned)(J - J_whole) < (unsigned)(I - J_whole);
    if (!full) {
      const int k_lo = J * BLK + 32 * kh, k_hi = k_lo + 31;
      const int q_lo = qbase, q_hi = qbase + 31;
      full = J >= 0 && k_hi <= q_lo && k_lo >= p0 && (!windowed || k_lo >= q_hi - p.w + 1);
      // no query of the group sees any of the 32 keys: later than all of them, padding, a skipped list
      // entry, or (plain window) wholly below the window: nothing to compute
      if (J < 0 || k_lo > q_hi || k_hi < p0 || (!EQ15 && windowed && k_hi < q_lo - p.w + 1)) return;
    }
    bf16x8 kf[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kf[kk] = *reinterpret_cast<const bf16x8 *>(ks + koff[kk]);
    bf16x8 vf[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const uint16_t *a0 = vs + 16 * t * D + voff[mb];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * D));
        vf[t][mb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    f32x16 s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], sinit, 0, 0, 0);
#pragma unroll
    for (int kk = 1; kk < 4; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
    if (!full) mask(J, windowed, s);
    // The exponentials are taken once: against the current reference, unless a row of the wavefront has
    // met no visible key yet (then the reference is placed first); a row sum that ran away repeats the
    // pass after raising the reference, which cannot run away again.
    bf16x8 pf[2];
    float tsum;
    bool placed = __any(fresh);
#pragma unroll 1
    for (;;) {
      if (placed) move_ref(s);
      tsum = expo(s, pf);
      if (placed || !__any(!(tsum <= kSumLimit4))) break;
      placed = true;
    }
    l_run += tsum;
    pv(vf, pf);
    if (hp) {
      bf16x8 pl[2];
      expo_lo(s, pf, pl);
      pv(vf, pl);
    }
  };

  // Closes a branch: the two wavefronts of a query group hold partial (reference, row sum, output)
  // triples over disjoint key halves.  Each hands the channel block it does not keep (32*(1-kh) ..)
  // to its partner through the staging rows just consumed (4 KB per wavefront) and merges the
  // partner's part of the block it keeps.  Leaves the normalised 32 rows x 32 channels (block kh) in
  // `fin` and returns the lse (natural log).  kx, vx: the tile buffers free at this point.
  f32x16 fin;
  auto close_branch = [&](uint16_t *kx, uint16_t *vx) __attribute__((always_inline)) -> float {
    __syncthreads();  // every wavefront is past its operand reads of kx, vx: they become exchange space
    float *area = reinterpret_cast<float *>(wv < 2 ? kx : vx);       // 2 wavefronts x 4 KB per buffer
    float *mine = area + (wv & 1) * 1024;                            // [16][64] floats
    const int pw = wv ^ 2;                                           // partner: same query group, other key half
    const float *theirs = reinterpret_cast<const float *>(pw < 2 ? kx : vx) + (pw & 1) * 1024;
    const float l_mine = l_run + __shfl_xor(l_run, 32);
    if (kh == 0) {
#pragma unroll
      for (int i = 0; i < 16; ++i) mine[i * 64 + lane] = oacc[1][i];
      fin = oacc[0];
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) mine[i * 64 + lane] = oacc[0][i];
      fin = oacc[1];
    }
    if (lh == 0) {
      xch_s[wv][0][lq] = fresh ? kNegInf : m_ref;
      xch_s[wv][1][lq] = l_mine;
    }
    __syncthreads();
    const float m_b = xch_s[pw][0][lq];
    const float l_b = xch_s[pw][1][lq];
    const float m_a = fresh ? kNegInf : m_ref;
    const float m = fmaxf(m_a, m_b);
    const float fa = m_a == kNegInf ? 0.0f : __builtin_amdgcn_exp2f(m_a - m);
    const float fb = m_b == kNegInf ? 0.0f : __builtin_amdgcn_exp2f(m_b - m);
    const float l_tot = l_mine * fa + l_b * fb;
    const bool ok = q_ok && l_tot > 0.0f;
    const float inv = ok ? 1.0f / l_tot : 0.0f;
    const float ga = fa * inv, gb = fb * inv;
#pragma unroll
    for (int i = 0; i < 16; ++i) fin[i] = fin[i] * ga + theirs[i * 64 + lane] * gb;
    __syncthreads();  // the partner has read this wavefront's rows: they may be refilled
    return ok ? (m + __log2f(l_tot)) * kLn2 : 0.0f;
  };

  // ---- walk over the tile list ----
  f32x16 ost;  // normalised short-term output (this wavefront's channel block), parked during the long-term walk
  float lse_st = 0.0f;
  reset();
  // Three buffer pairs, tiles requested two steps ahead: a tile's global->LDS loads have two whole
  // steps to land (the L2 latency under load is longer than one step of a wavefront).
  // step t: request tile t+2 into the pair that held tile t-1 (every wavefront is past its reads of it:
  // barrier at the end of step t-1), process tile t, wait for this wavefront's own loads of tile t+1
  // (the four of tile t+2 stay in flight), barrier.
  int J_cur = first_J;
  int J_n1 = list_at(1);
  int J_n2 = list_at(2);
  if (n_all > 1) {
    stage(Kh, k_lane, 64u, Ks1, J_n1);
    stage(Vh, v_lane, 0u, Vs1, J_n1);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm4(4));
  } else {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm4(0));
  }
  __syncthreads();  // tile 0 and the gate weights are in LDS
  auto step = [&](int t, uint16_t *k_cur, uint16_t *v_cur, uint16_t *k_fill, uint16_t *v_fill) __attribute__((always_inline)) {
    const bool more = t + 2 < n_all;
    if (more) {
      stage(Kh, k_lane, 64u, k_fill, J_n2);
      stage(Vh, v_lane, 0u, v_fill, J_n2);
    }
    tile(k_cur, v_cur, J_cur, t < n_st);
    J_cur = J_n1;
    J_n1 = J_n2;
    if (((t + 3) & 63) == 0 && t + 3 < n_all) tl = list_chunk((t + 3) >> 6);  // (once per 64 tiles)
    J_n2 = list_at(t + 3);
    if (t + 1 == n_st) {  // the short-term tiles are done (the merge has its own barriers)
      lse_st = close_branch(k_cur, v_cur);
      ost = fin;
      reset();
      set_ref(0.0f);
    }
    if (more) __builtin_amdgcn_s_waitcnt(vmcnt_imm4(4));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm4(0));
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 3) {
    step(t, Ks0, Vs0, Ks2, Vs2);
    if (t + 1 < n_all) step(t + 1, Ks1, Vs1, Ks0, Vs0);
    if (t + 2 < n_all) step(t + 2, Ks2, Vs2, Ks1, Vs1);
  }
  const float lse_lt = close_branch(Ks0, Vs0);

  // ---- epilogue: gate (Eq. 18-19) and stores of this wavefront's 32 rows x 32 channels ----
  // fin[4*g + e] (and ost): channel 32*kh + 8*g + 4*lh + e of row qbase + lq.  The tiles leave through
  // LDS (this wavefront's own 4 KB of the staging buffers, free now) as 128-byte (fp32) or 64-byte
  // (bf16) row segments.
  int el = lane;  // opaque copy: keeps the store addressing out of the registers of the tile loop
  asm volatile("" : "+v"(el));
  const int elq = el & 31, elh = el >> 5;
  float *xa = reinterpret_cast<float *>(wv < 2 ? Ks0 : Vs0) + (wv & 1) * 1024;  // 4 KB
  auto store_f32_rows = [&](float *dst, const f32x16 &acc) __attribute__((always_inline)) {
    // write: row elq, 16-byte chunk (2*g + elh) of the 8 chunks of its 128-byte segment, XOR-swizzled
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int chunk = 2 * g + elh;
      *reinterpret_cast<float4 *>(xa + elq * 32 + ((chunk ^ (elq & 7)) * 4)) =
          make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
    }
    // read: 8 lanes per row, 8 rows per instruction
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = 8 * i + (el >> 3), c = el & 7;
      const float4 v = *reinterpret_cast<const float4 *>(xa + rr * 32 + ((c ^ (rr & 7)) * 4));
      const int grow = qbase + rr;
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
      const f32x4_t vv = {v.x, v.y, v.z, v.w};
      if (grow < p.L)
        __builtin_nontemporal_store(vv, reinterpret_cast<f32x4_t *>(dst + head + (size_t)grow * D + 32 * kh + 4 * c));
    }
  };
  auto store_bf16_rows = [&](uint16_t *dst, auto o4) __attribute__((always_inline)) {
    uint16_t *pt = reinterpret_cast<uint16_t *>(xa);  // 32 rows of 64 bytes
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 pk;
      pk.x = pack2_bf16(o4(g, 0), o4(g, 1));
      pk.y = pack2_bf16(o4(g, 2), o4(g, 3));
      // 16-byte chunk g of the row's 4 (8 channels); this lane fills half elh of it
      *reinterpret_cast<uint2 *>(pt + elq * 32 + ((g ^ (elq & 3)) * 8) + 4 * elh) = pk;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rr = 16 * i + (el >> 2), c = el & 3;
      const uint4 v = *reinterpret_cast<const uint4 *>(pt + rr * 32 + ((c ^ (rr & 3)) * 8));
      const int grow = qbase + rr;
      if (grow < p.L) *reinterpret_cast<uint4 *>(dst + head + (size_t)grow * D + 32 * kh + 8 * c) = v;
    }
  };
  const size_t lrow = (size_t)bh * p.L + iq;
  if (dense) {
    store_bf16_rows(O, [&](int g, int e) { return fin[4 * g + e]; });
    if (iq < p.L && lh == 0 && kh == 0 && lse_lt_out) lse_lt_out[lrow] = lse_lt;
    return;
  }
  float z = 0.0f;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int d0 = 32 * kh + 8 * g + 4 * lh;
    const float4 a = *reinterpret_cast<const float4 *>(gate_s + d0);
    const float4 b = *reinterpret_cast<const float4 *>(gate_s + D + d0);
    z = fmaf(a.x, fin[4 * g], z);
    z = fmaf(a.y, fin[4 * g + 1], z);
    z = fmaf(a.z, fin[4 * g + 2], z);
    z = fmaf(a.w, fin[4 * g + 3], z);
    z = fmaf(b.x, ost[4 * g], z);
    z = fmaf(b.y, ost[4 * g + 1], z);
    z = fmaf(b.z, ost[4 * g + 2], z);
    z = fmaf(b.w, ost[4 * g + 3], z);
  }
  z += __shfl_xor(z, 32);
  if (lh == 0) xch_s[wv][2][lq] = z;
  __syncthreads();
  // both wavefronts of the pair add the two partial sums in the same order: the same alpha bit for bit
  z = xch_s[qg][2][lq] + xch_s[qg + 2][2][lq];
  z += gate_b ? gate_b[h] : 0.0f;
  const float alpha = q_ok ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
  if (o_lt_out) {
    store_f32_rows(o_lt_out, fin);
    store_f32_rows(o_st_out, ost);
  }
  store_bf16_rows(O, [&](int g, int e) { return alpha * fin[4 * g + e] + (1.0f - alpha) * ost[4 * g + e]; });
  if (iq < p.L && lh == 0 && kh == 0) {
    if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
    if (lse_st_out) lse_st_out[lrow] = lse_st;
  }
}

void launch_fwd_mfma4(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  const unsigned grid = (unsigned)(p.B * p.H * p.nq);
  auto u16 = [](const void *x) { return reinterpret_cast<const uint16_t *>(x); };
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, u16(a.Q), u16(a.K), u16(a.V), a.valid_len, a.sel,
                       a.gate_w, a.gate_b, (uint16_t *)a.O, (float *)a.o_lt, (float *)a.o_st, a.lse_lt, a.lse_st,
                       a.dense, p);
  };
  const bool eq15 = p.sblk != 0 && !a.dense;
  const bool sub = eq15 && p.sblk < p.b;  // mask block smaller than the tile
  if (sub) go(fwd_mfma4_kernel<true, true>);
  else if (eq15) go(fwd_mfma4_kernel<true, false>);
  else go(fwd_mfma4_kernel<false, false>);
}

}  // namespace blossom

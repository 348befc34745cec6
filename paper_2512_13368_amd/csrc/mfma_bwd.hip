// Backward on the matrix cores for bf16, d = 64, block size 32 or 64: dQ (query-block
// stationary) and dK/dV (key-block stationary), chain rule through Eq. 1 and Eq. 16-19 with
// the selection held fixed.
//
// The upstream gradient of branch x is dO_x = a_x*dO + dz*Wg_x (a_lt = alpha, a_st = 1-alpha;
// gate backward).  The per-row pass rounds it to bf16 ONCE and derives the row constant
// c_x = dO_x.o_x from the same rounded values; then
//   dS_ij = P_ij * (dO_x,i.v_j - c_x,i),   dV_j = sum_i P_ij dO_x,i,   dK_j = sum_i dS_ij q_i,
//   dQ_i = sum_j dS_ij k_j
// is the exact softmax backward of the rounded gradient: the cancellation that rows with one
// or two keys rely on (dO_x.v_j = c_x when P = 1) survives, and the kernels are left with one
// exponential, one multiply and the bf16 conversions per score.
//
// Accumulators start at minus a per-row constant, so the MFMA result is directly what the next
// step needs: the exponent S'' = c*q.k - lse*log2(e) (Q or K pre-multiplied by c =
// scale*log2(e)) and dO_x,i.v_j - c_x,i.  The constants arrive as three-term bf16 splits (exact).
// dK/dV, where they change with every query tile, broadcasts them into the accumulator by one
// extra matrix instruction (ones x split); dQ, where a lane keeps its row for the whole walk,
// holds them as two 16-register blocks that the first matrix instruction of each product
// takes as its C operand.  Either way no per-element VALU initialisation is needed.  (Reading
// the dK/dV constants from LDS straight into a C block was measured slower: that kernel
// already issues 25 LDS reads per 18 matrix instructions.)  Probabilities and dS leave the accumulator
// registers as the B operand of the next product without moving between lanes; the matching
// A operands (K^T, Q^T, dO_x^T) come from LDS through the transposing ds_read_b64_tr_b16.
// Query blocks whose rows may see only a few keys (large probabilities) feed P and dS as
// two-term bf16 sums.
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

using namespace mfma;

namespace {

// Per-lane LDS BYTE offsets of the two operand read patterns for a tile staged with swz().
// Kept in bytes and passed through an empty asm by the kernels, so that "tile base + offset +
// constant" is formed next to each read and the constant folds into the instruction's immediate.
struct ReadOffsets {
  int row[4];  // row-per-lane 16-byte reads: slab kk; add 2*32*unit*D
  int tr[2];   // transposing 8-byte reads: M-block mb; add 2*(32*unit + 16*t)*D
  int tr8[2];  // the same for the read 8 rows further down (row bit 3 set: another swizzle)
};

__device__ __forceinline__ ReadOffsets read_offsets(int lane)
{
  ReadOffsets o;
  const int lq = lane & 31, lh = lane >> 5, r16 = lane & 15, g1 = (lane >> 4) & 1;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) o.row[kk] = 2 * (lq * D + (((2 * kk + lh) ^ swz(lq)) * 8));
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
  {
    const int row = 4 * lh + (r16 >> 2);  // rows row and row + 8 of a 16-row contraction slab
    const int chunk = 4 * mb + 2 * g1 + ((r16 & 3) >> 1);
    o.tr[mb] = 2 * (row * D + ((chunk ^ swz(row)) * 8) + 4 * (r16 & 1));
    o.tr8[mb] = 2 * ((row + 8) * D + ((chunk ^ swz(row + 8)) * 8) + 4 * (r16 & 1));
  }
  return o;
}

// Direct global->LDS staging of one tile (BLK rows x 128 bytes): each wavefront moves 4 x 1 KB.
// A tile's rows are contiguous in memory and the LDS copy keeps the 128-byte row pitch, so one
// uniform base (SGPRs), one per-lane byte offset and the same immediate on the global and the
// LDS side address the four 8-row slices.
template <int BLK>
struct Stager {
  int wv, ld_row;
  bool ragged;
  int L, NB;
  unsigned lane_off;  // bytes: (ld_row, chunk) of this lane inside a tile, 8-row slices 0 and 2
  unsigned lane_odd;  // the same for slices 1 and 3 (row bit 3 set: another swizzle)
  __device__ __forceinline__ void init(int wv_, int lane, int L_, int NB_)
  {
    wv = wv_;
    L = L_;
    NB = NB_;
    ld_row = 32 * wv + (lane >> 3);
    ragged = L % BLK != 0;
    // LDS chunk position lane&7 holds chunk (lane&7)^swz(row)
    lane_off = (unsigned)(ld_row * D + ((lane & 7) ^ swz(ld_row)) * 8) * 2u;
    lane_odd = (unsigned)(ld_row * D + ((lane & 7) ^ swz(ld_row + 8)) * 8) * 2u;
  }
  // src_head: first element of the (row, head) slice of the tensor
  __device__ __forceinline__ void stage(const uint16_t *src_head, uint16_t *dst_tile, int blk) const
  {
    constexpr int TILE = BLK * D;
    const char *src = reinterpret_cast<const char *>(src_head) + (size_t)max(blk, 0) * (TILE * 2);  // uniform (block -1: a skipped list entry, every key masked)
    lds_void *dst = (lds_void *)(dst_tile + 32 * wv * D);
    if (!ragged || blk != NB - 1) {
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 1024, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 2048, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 3072, 0);
    } else {  // last, partial block: rows past the end are clamped (always masked)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int over = max(0, blk * BLK + ld_row + 8 * u - (L - 1));
        const unsigned off = ((u & 1) ? lane_odd : lane_off) + (unsigned)((8 * u - over) * D * 2);
        __builtin_amdgcn_global_load_lds((glb_void *)(src + off), (lds_void *)(dst_tile + (32 * wv + 8 * u) * D), 16, 0, 0);
      }
    }
  }
};

// off: byte offset inside the tile
__device__ __forceinline__ bf16x8 lds_row(const uint16_t *tile, int off)
{
  return *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const char *>(tile) + off);
}

__device__ __forceinline__ bf16x8 lds_tr(const uint16_t *tile, int off, int off8)
{
  const char *a = reinterpret_cast<const char *>(tile);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + off));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + off8));
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

// Stores 2 x 16 accumulators (d x rows, transposed) as bf16, scaled, through LDS: the wavefront's 32 rows
// (this lane: row lane%32, channels
// 32*mb + 8*g + 4*(lane/32) + e in acc[mb][4*g + e]) are written into its own 4 KB of staging rows
// (free once the walk is over; chunks XOR-swizzled against bank conflicts) and leave as whole
// 128-byte rows, 8 rows per store instruction, non-temporal (nothing in this library reads the
// gradients back).  Rows that are not kept are stored as zeros, rows at or past rows_left not at all.
// `unrope` (dQ and dK when the caller's Q and K went through the rotary position embedding): the rows
// are rotated back first; a lane's four consecutive channels are two whole channel pairs.  m_row0 is
// the position of the first of the 32 rows, L the sequence length (rows past it are never stored).
__device__ __forceinline__ void store_rows_bf16(uint16_t *dst_row0, int rows_left, uint16_t *pt, const f32x16 (&acc)[2],
                                                float scale, bool keep, const KParams &p, bool unrope = false, int m_row0 = 0)
{
  int el;  // the lane id, rebuilt here so that none of the addressing below is computed ahead of the walk
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(el));
  const int elq = el & 31, elh = el >> 5;
  const float sc = keep ? scale : 0.0f;
  const bool rot = unrope && p.rope_cos != nullptr;
  const int m = min(m_row0 + elq, p.L - 1);
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float v0 = acc[mb][4 * g], v1 = acc[mb][4 * g + 1], v2 = acc[mb][4 * g + 2], v3 = acc[mb][4 * g + 3];
      if (rot) {
        const int pair = 16 * mb + 4 * g + 2 * elh;  // channels 32*mb + 8*g + 4*elh + (0..3)
        unrope_pair(p, m, pair, D / 2, v0, v1);
        unrope_pair(p, m, pair + 1, D / 2, v2, v3);
      }
      uint2 pk;
      pk.x = pack2_bf16(v0 * sc, v1 * sc);
      pk.y = pack2_bf16(v2 * sc, v3 * sc);
      const int chunk = 4 * mb + g;  // 16-byte chunk of the row; this lane fills half elh of it
      *reinterpret_cast<uint2 *>(pt + elq * D + ((chunk ^ (elq & 7)) * 8) + 4 * elh) = pk;
    }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rr = 8 * i + (el >> 3), c = el & 7;
    const uint4 v = *reinterpret_cast<const uint4 *>(pt + rr * D + ((c ^ (rr & 7)) * 8));
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t vv = {v.x, v.y, v.z, v.w};
    if (rr < rows_left) __builtin_nontemporal_store(vv, reinterpret_cast<u32x4_t *>(dst_row0 + (size_t)rr * D + 8 * c));
  }
}

constexpr int kFewKeys = 32;    // rows seeing fewer keys than this get two-term bf16 operands

// ones[.][0..2] in the half of the wavefront that holds contraction slots 0..7: multiplied with a
// three-term split it broadcasts the split's value along the other dimension of the tile
__device__ __forceinline__ bf16x8 ones3(int lh)
{
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)((lh == 0 && e < 3) ? 1.0f : 0.0f);
  return o;
}

// a packed split (hi | mid << 16, lo) as an MFMA operand (slots 0..2; lanes of the other half
// meet zeros of ones3 and may hold anything finite)
__device__ __forceinline__ bf16x8 split_operand(uint32_t x, uint32_t y)
{
  const uint4 raw = make_uint4(x, y, 0u, 0u);
  return __builtin_bit_cast(bf16x8, raw);
}

}  // namespace

// =============================================================================================
// dQ: one workgroup per (row, head, query block), one wavefront per 32 query rows.
//   per 32-key unit:  S''^T = K (cQ)^T - lse2       (keys x queries, lane owns a query column)
//                     G^T   = V dO_x^T - c_x
//                     dS^T  = 2^S'' * G^T  -> bf16 -> B operand
//                     dQ^T += K^T dS^T      (K^T through the transposing LDS read)
// EQ15: the short-term mask is all of Eq. 15, with mask block BLK or (SUB) a power of two below it;
// compile-time variants of both kernels, so that the plain window keeps its code.
// =============================================================================================
// (pid: the workgroup's index among the dQ workgroups of the launch; Ks0..Vs1: four staging tiles of BLK*D halfwords
// in LDS, 1 KB aligned, distinct objects)
template <int BLK, bool EQ15, bool SUB>
__device__ __forceinline__ void bwd_dq_body(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int *__restrict__ valid_len, const int *__restrict__ sel, const uint16_t *__restrict__ g_lt,
    const uint16_t *__restrict__ g_st, const uint4 *__restrict__ rowI_lt, const uint4 *__restrict__ rowI_st,
    const uint16_t *__restrict__ dO, const float4 *__restrict__ rowstat, const float *__restrict__ gate_w,
    const float *__restrict__ o_lt, const float *__restrict__ o_st, uint16_t *__restrict__ dQ, KParams p, unsigned pid,
    uint16_t *Ks0, uint16_t *Ks1, uint16_t *Vs0, uint16_t *Vs1)
{
  constexpr int UNITS = BLK / 32;
  constexpr int TILE = BLK * D;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: MFMA regions must be scalar branches
  const int lq = lane & 31, lh = lane >> 5;
  const unsigned vid = xcd_remap(pid, (unsigned)(p.B * p.H * p.NB));
  const int bh = (int)(vid / p.NB);
  const int I = p.NB - 1 - (int)(vid % p.NB);
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int q0 = I * BLK + 32 * wv;
  const int iq = q0 + lq;
  const bool q_ok = iq < p.L && iq >= p0;
  const size_t head = (size_t)bh * p.L * D;
  const size_t rowoff = head + (size_t)min(iq, p.L - 1) * D;
  const size_t lrow = (size_t)bh * p.L + min(iq, p.L - 1);

  f32x16 dq[2];
#pragma unroll
  for (int i = 0; i < 16; ++i) { dq[0][i] = 0.0f; dq[1][i] = 0.0f; }
  if (min((I + 1) * BLK, p.L) <= p0) {  // no valid query: gradients are zero
    zero_rows(dQ + head, q0, 32, p.L, lane);
    return;
  }

  const float c2 = p.scale * kLog2e;
  bf16x8 qf[4], gf[4], gf_next[4];
  load_frags(Q + rowoff, lh, c2, qf);
  load_frags(g_st + rowoff, lh, 1.0f, gf);       // the walk starts with the window tiles
  load_frags(g_lt + rowoff, lh, 1.0f, gf_next);
  // per-row constants (pad rows carry an exponent of -1e30: every probability of the column is zero)
  const uint4 ri_st = rowI_st[lrow];
  const uint4 ri_lt = rowI_lt[lrow];
  // s_init, g_init: -lse2[i] and -c_x[i] of this lane's row in every accumulator slot.  The
  // first matrix instruction of each product takes them as its C operand, so the logits and
  // dP - c_x leave the matrix cores with the row terms already applied.
  f32x16 s_init, g_init;
  auto set_init = [&](uint32_t sx, uint32_t sy, uint32_t cx, uint32_t cy) __attribute__((always_inline)) {
    const float a = unsplit3(sx, sy), b = unsplit3(cx, cy);
#pragma unroll
    for (int i = 0; i < 16; ++i) { s_init[i] = a; g_init[i] = b; }
    asm volatile("" : "+v"(s_init), "+v"(g_init));  // register blocks, not one value copied at each use
  };

  // ---- tile list: window blocks, then the selection list up to its last valid entry ----
  const int J_first = p0 / BLK;
  const int lowpos = I * BLK - (p.w - 1);
  int J_lo = lowpos <= 0 ? 0 : lowpos / BLK;
  // SUB: the mask block of Eq. 15 is a power of two below BLK.  The mask-block distances 2^r below
  // one tile then reach into block I - 1, which joins the window range; the larger ones land on
  // the blocks I - 2^r' as before; every short-term tile is masked element by element.
  constexpr bool sub = EQ15 && SUB;
  const int sub_sh = sub ? __builtin_ctz((unsigned)p.sblk) : 0;
  if (sub) J_lo = min(J_lo, I - 1);
  J_lo = max(J_lo, J_first);
  // With the full short-term mask (Eq. 15) the blocks I - 2^r below the window
  // range follow the window blocks: r = r0 .. r0 + n_pow - 1.
  const int n_win = I - J_lo + 1;
  int n_st = n_win, r0 = 0;
  if (EQ15 && I > J_first) {
    const int d_win = I - J_lo;                                      // largest block distance inside the window range
    r0 = d_win == 0 ? 0 : 32 - __builtin_clz((unsigned)d_win);       // smallest r with 2^r > d_win
    const int r_max = 31 - __builtin_clz((unsigned)(I - J_first));   // largest r with I - 2^r >= J_first
    n_st += max(0, r_max - r0 + 1);
  }
  int n_lt = 0;
  bool lt_few = true;  // the selected past blocks hold fewer than kFewKeys valid keys
  const int *my_sel = sel + ((size_t)bh * p.NB + I) * p.k;
  // (entries outside [0, NB) are skipped wherever they stand: the walk runs up to the last valid
  // entry, an invalid one in between costs one tile with every key masked)
  for (int e0 = 0; e0 < p.k; e0 += 64) {
    const int e = e0 + lane;
    const int J = e < p.k ? my_sel[e] : -1;
    const bool ok = J >= 0 && J < p.NB;
    const unsigned long long okm = __ballot(ok);
    if (okm != 0ull) n_lt = e0 + 64 - __builtin_clzll(okm);
    const int vcount = min((J + 1) * BLK, p.L) - max(J * BLK, p0);
    if (__ballot(ok && J < I && vcount >= kFewKeys) != 0ull) lt_few = false;
  }
  // Rows with only a few keys: dq is a sum of a few large dS*k terms that nearly cancel, so the
  // bf16 rounding of dS would dominate it.  Such wavefronts feed dS as a two-term bf16 sum.
  const int hp_st = __builtin_amdgcn_readfirstlane((int)(p.w < kFewKeys || q0 - p0 + 1 < kFewKeys));
  const int hp_lt = __builtin_amdgcn_readfirstlane((int)lt_few);
  const int n_all = n_st + n_lt;
  // For those rows the bf16 rounding of dO_x itself would show as well (dS is large, and the
  // small projections dO_x.(v_j - o) lose relative accuracy): the residual dO_x - bf16(dO_x) is
  // rebuilt from dO, alpha, dz and the gate weights exactly as the per-row pass formed it, and
  // enters as a second B operand; the row constant gains the matching residual.o_x.
  bf16x8 gl[4], gl_next[4];
  uint32_t c1_st_x = ri_st.z, c1_st_y = ri_st.w, c1_lt_x = ri_lt.z, c1_lt_y = ri_lt.w;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int e = 0; e < 8; ++e) { gl[kk][e] = (__bf16)0.0f; gl_next[kk][e] = (__bf16)0.0f; }
  if (hp_st | hp_lt) {
    const float4 st = rowstat[lrow];
    const float *wrow = gate_w + (size_t)(bh % p.H) * 2 * D;
    float corr_st = 0.0f, corr_lt = 0.0f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(dO + rowoff + 16 * kk + 8 * lh);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int dd = 16 * kk + 8 * lh + e;
        const float g = (e & 1) ? bf_hi(w[e >> 1]) : bf_lo(w[e >> 1]);
        const float full_l = fmaf(st.x, g, st.y * wrow[dd]);
        const float full_s = fmaf(1.0f - st.x, g, st.y * wrow[D + dd]);
        const __bf16 lo_l = (__bf16)(full_l - bf16_to_f32(f32_to_bf16(full_l)));
        const __bf16 lo_s = (__bf16)(full_s - bf16_to_f32(f32_to_bf16(full_s)));
        gl_next[kk][e] = lo_l;
        gl[kk][e] = lo_s;
        corr_lt = fmaf((float)lo_l, o_lt[rowoff + dd], corr_lt);
        corr_st = fmaf((float)lo_s, o_st[rowoff + dd], corr_st);
      }
    }
    corr_lt += __shfl_xor(corr_lt, 32);
    corr_st += __shfl_xor(corr_st, 32);
    const uint2 ns = split3(unsplit3(ri_st.z, ri_st.w) - corr_st);
    const uint2 nl = split3(unsplit3(ri_lt.z, ri_lt.w) - corr_lt);
    if (q_ok) {
      c1_st_x = ns.x; c1_st_y = ns.y; c1_lt_x = nl.x; c1_lt_y = nl.y;
    }
  }
  set_init(ri_st.x, ri_st.y, c1_st_x, c1_st_y);
  __syncthreads();
  // Block id of tile t: window blocks by arithmetic, selected blocks by a scalar load from the
  // selection row (uniform address), issued a whole tile before its value is needed.
  auto tile_of = [&](int t) -> int {
    const int e = __builtin_amdgcn_readfirstlane(t - n_st);
    typedef const int __attribute__((address_space(4))) *const_int_ptr;  // read-only: loads become scalar
    if (e >= 0) return ((const_int_ptr)my_sel)[e];  // raw: may be outside [0, NB), see list_entry
    if (!EQ15) return J_lo + t;
    return t < n_win ? J_lo + t : I - (1 << (r0 + t - n_win));
  };

  // a raw tile-list value when it is consumed (a whole tile after its scalar load was issued): entries
  // outside [0, NB) become -1, a tile whose keys are all masked
  auto list_entry = [&](int raw) -> int { return (unsigned)raw < (unsigned)p.NB ? raw : -1; };

  Stager<BLK> sg;
  sg.init(wv, lane, p.L, p.NB);
  const uint16_t *k_lane = K + head;  // (row, head) slices; the stager adds block and lane offsets
  const uint16_t *v_lane = V + head;
  ReadOffsets ro = read_offsets(lane);

  auto tile_body = [&](const uint16_t *ks, const uint16_t *vs, int J, bool short_term) __attribute__((always_inline)) {
    asm volatile("" : "+v"(ro.row[0]), "+v"(ro.row[1]), "+v"(ro.row[2]), "+v"(ro.row[3]), "+v"(ro.tr[0]), "+v"(ro.tr[1]), "+v"(ro.tr8[0]), "+v"(ro.tr8[1]));
    const bool hp = (short_term ? hp_st : hp_lt) != 0;
    // band-masked by the window, unless Eq. 15 shows the whole block (power-of-two block distance)
    const bool windowed = short_term && !(EQ15 && !sub && is_pow2(I - J));
    const bool masked = windowed || J == I || J * BLK < p0;
    int wlo = iq - p.w + 1;
    if (EQ15 && iq >= p.last_lo) wlo = min(wlo, p.last_lo);  // third case of Eq. 15: the last block is visible to its own rows
    const int lo = windowed ? max(p0, wlo) : p0;
    const unsigned span = (unsigned)(iq - lo);
    const bool any = iq >= lo;
#pragma unroll
    for (int s = 0; s < UNITS; ++s) {
      f32x16 sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(ks, 2 * 32 * s * D + ro.row[0]), qf[0], s_init, 0, 0, 0);
      f32x16 gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(vs, 2 * 32 * s * D + ro.row[0]), gf[0], g_init, 0, 0, 0);
#pragma unroll
      for (int kk = 1; kk < 4; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(ks, 2 * 32 * s * D + ro.row[kk]), qf[kk], sacc, 0, 0, 0);
        gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(vs, 2 * 32 * s * D + ro.row[kk]), gf[kk], gacc, 0, 0, 0);
      }
      if (hp) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(vs, 2 * 32 * s * D + ro.row[kk]), gl[kk], gacc, 0, 0, 0);
      }
      if (masked) {
        const int base = J * BLK + 32 * s + 4 * lh;
        if (sub && windowed && J < J_lo && J * BLK >= p0) {
          // a block I - 2^r' below the window range, all of it valid: visible iff row and key share
          // the mask block within their tiles (no window, no last-block key, one possible power of two)
          const int qo = iq & (BLK - 1);
          const int kb = 32 * s + 4 * lh;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int ko = kb + 8 * (i >> 2) + (i & 3);
            sacc[i] = (((qo ^ ko) >> sub_sh) == 0 && q_ok) ? sacc[i] : kNegInf;
          }
        } else if (sub && windowed) {
          // window range, or (valid, causal and) a power-of-two mask-block distance, or a last-block key
          const unsigned cspan = (unsigned)(iq - p0);
          const bool cany = iq >= p0;
          const int qmb = iq >> sub_sh;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = base + 8 * (i >> 2) + (i & 3);
            const int x = qmb - (key >> sub_sh);
            const bool far = cany & ((unsigned)(key - p0) <= cspan) & ((x > 0 && (x & (x - 1)) == 0) | (key >= p.last_lo));
            const bool vis = (any & ((unsigned)(key - lo) <= span)) | far;
            sacc[i] = vis ? sacc[i] : kNegInf;
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = base + 8 * (i >> 2) + (i & 3);
            const bool vis = any & ((unsigned)(key - lo) <= span);
            sacc[i] = vis ? sacc[i] : kNegInf;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = __builtin_amdgcn_exp2f(sacc[i]) * gacc[i];  // dS
      bf16x8 dsf[2];
      to_operand(sacc, dsf);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          dq[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(ks, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), dsf[t],
                                                           dq[mb], 0, 0, 0);
      if (hp) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] -= (float)dsf[i >> 3][i & 7];
        to_operand(sacc, dsf);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
            dq[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(ks, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), dsf[t],
                                                             dq[mb], 0, 0, 0);
      }
    }
  };

  int J_cur = list_entry(tile_of(0));
  int J_nxt = list_entry(tile_of(min(1, n_all - 1)));
  sg.stage(k_lane, Ks0, J_cur);
  sg.stage(v_lane, Vs0, J_cur);
  __syncthreads();
  auto step = [&](int t, uint16_t *k_fill, uint16_t *v_fill, const uint16_t *k_cur, const uint16_t *v_cur)
                  __attribute__((always_inline)) {
    const int J_after = tile_of(min(t + 2, n_all - 1));  // consumed at the end of this step
    if (t + 1 < n_all) {
      sg.stage(k_lane, k_fill, J_nxt);
      sg.stage(v_lane, v_fill, J_nxt);
    }
    if (t == n_st) {  // the long-term tiles start: switch to that branch's gradient and constants
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        gf[kk] = gf_next[kk];
        gl[kk] = gl_next[kk];
      }
      set_init(ri_lt.x, ri_lt.y, c1_lt_x, c1_lt_y);
    }
    tile_body(k_cur, v_cur, J_cur, t < n_st);
    J_cur = J_nxt;
    J_nxt = list_entry(J_after);
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Ks1, Vs1, Ks0, Vs0);
    if (t + 1 < n_all) step(t + 1, Ks0, Vs0, Ks1, Vs1);
  }
  {  // (every wavefront is past the last barrier of the walk: the staging rows are free)
    const int row0 = I * BLK + 32 * wv;
    store_rows_bf16(dQ + head + (size_t)row0 * D, p.L - row0, Ks0 + wv * 32 * D, dq, p.scale, q_ok, p, true, row0);
  }
}

// =============================================================================================
// dK, dV: one workgroup per (row, head, key block), one wavefront per 32 key rows; walks the
// query blocks whose window reaches the key block, then those that selected it (inverse list).
//   per 32-query unit:  S'' = Q (cK)^T - lse2[i]   (queries x keys, lane owns a key column)
//                       G   = dO_x V^T - c_x[i]
//                       P = 2^S'',  dS = P*G
//                       dV^T += dO_x^T P,  dK^T += Q^T dS
// =============================================================================================

template <int BLK, bool EQ15, bool SUB>
__device__ __forceinline__ void bwd_dkv_body(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int *__restrict__ valid_len, const uint16_t *__restrict__ g_lt, const uint16_t *__restrict__ g_st,
    const uint4 *__restrict__ rowI_lt, const uint4 *__restrict__ rowI_st, const int *__restrict__ offs,
    const int *__restrict__ items, const uint16_t *__restrict__ dO, const float4 *__restrict__ rowstat,
    const float *__restrict__ gate_w, const float *__restrict__ o_lt, const float *__restrict__ o_st,
    uint16_t *__restrict__ dK, uint16_t *__restrict__ dV, KParams p, unsigned pid, uint16_t *Qs0, uint16_t *Qs1,
    uint16_t *Gs0, uint16_t *Gs1, uint4 (*rc_s)[BLK])
{
  // (rc_s: per-row constants of the staged query tile: splits of -lse2 (x, y) and of -c_x (z, w))
  constexpr int UNITS = BLK / 32;
  constexpr int TILE = BLK * D;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31, lh = lane >> 5;
  const unsigned vid = xcd_remap(pid, (unsigned)(p.B * p.H * p.NB));
  const int bh = (int)(vid / p.NB);
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
    zero_rows(dK + head, J * BLK + 32 * wv, 32, p.L, lane);
    zero_rows(dV + head, J * BLK + 32 * wv, 32, p.L, lane);
    return;
  }
  const float c2 = p.scale * kLog2e;
  bf16x8 kf[4], vf[4];
  load_frags(K + rowoff, lh, c2, kf);
  load_frags(V + rowoff, lh, 1.0f, vf);
  const bf16x8 ones = ones3(lh);

  // ---- walk: window part I = J..I_hi, then the inverse selection list ----
  const long last_q = (long)J * BLK + (BLK - 1) + (p.w - 1);
  // SUB: the mask block of Eq. 15 is a power of two below BLK: block J + 1 joins the window range (the
  // mask-block distances below one tile reach it), every short-term tile is masked element by element.
  constexpr bool sub = EQ15 && SUB;
  const int sub_sh = sub ? __builtin_ctz((unsigned)p.sblk) : 0;
  int I_hi = (int)min((long)(p.NB - 1), last_q / BLK);
  if (sub) I_hi = max(I_hi, min(J + 1, p.NB - 1));
  // With the full short-term mask (Eq. 15) the query blocks J + 2^r above the
  // window range follow: r = r0 .. r0 + n_pow - 1.
  const int n_win = I_hi - J + 1;
  int n_st = n_win, r0 = 0;
  if (EQ15 && p.NB - 1 > J) {
    const int d_win = I_hi - J;                                       // largest block distance inside the window range
    r0 = d_win == 0 ? 0 : 32 - __builtin_clz((unsigned)d_win);        // smallest r with 2^r > d_win
    const int r_max = 31 - __builtin_clz((unsigned)(p.NB - 1 - J));   // largest r with J + 2^r <= NB - 1
    n_st += max(0, r_max - r0 + 1);
  }
  const int e_lo = offs[(size_t)bh * (p.NB + 1) + J];
  const int n_lt = offs[(size_t)bh * (p.NB + 1) + J + 1] - e_lo;
  const int n_all = n_st + n_lt;
  const int *my_items = items + (size_t)bh * p.NB * p.k + e_lo;
  // Query block of step t, with the few-keys flag of the list entries in bit kInvFewShift:
  // window blocks by arithmetic, list entries by a scalar load (uniform address), issued a
  // whole tile before the value is needed.
  auto entry_of = [&](int t) -> int {
    const int e = __builtin_amdgcn_readfirstlane(t - n_st);
    typedef const int __attribute__((address_space(4))) *const_int_ptr;  // read-only: loads become scalar
    if (e >= 0) return ((const_int_ptr)my_items)[e];
    if (!EQ15) return J + t;
    return t < n_win ? J + t : J + (1 << (r0 + t - n_win));
  };

  Stager<BLK> sg;
  sg.init(wv, lane, p.L, p.NB);
  const uint16_t *q_lane = Q + head;  // (row, head) slices; the stager adds block and lane offsets
  const uint16_t *gl_lane = g_lt + head;
  const uint16_t *gs_lane = g_st + head;
  ReadOffsets ro = read_offsets(lane);
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const uint4 pad_consts = make_uint4(0x0000f149u, 0u, 0u, 0u);  // -1e30 as (hi, 0, 0): probability zero

  // per-row constants of query block Iq for one branch (rows past the end: probability zero)
  auto row_consts = [&](int Iq, bool windowed) __attribute__((always_inline)) -> uint4 {
    uint4 r = pad_consts;
    if (tid < BLK) {
      const int i = Iq * BLK + tid;
      if (i < p.L) r = (windowed ? rowI_st : rowI_lt)[lbase + i];
    }
    return r;
  };

  auto tile_body = [&](const uint16_t *qs, const uint16_t *gsm, int par, int Iq, bool short_term, bool hp)
                       __attribute__((always_inline)) {
    // band-masked by the window, unless Eq. 15 shows the whole block (power-of-two block distance)
    const bool windowed = short_term && !(EQ15 && !sub && is_pow2(Iq - J));
    asm volatile("" : "+v"(ro.row[0]), "+v"(ro.row[1]), "+v"(ro.row[2]), "+v"(ro.row[3]), "+v"(ro.tr[0]), "+v"(ro.tr[1]), "+v"(ro.tr8[0]), "+v"(ro.tr8[1]));
    const bool masked = windowed || Iq == J || Iq * BLK < p0 || J * BLK < p0 || (Iq + 1) * BLK > p.L;
    // visible <=> key valid and lo_i <= i <= hi_i
    const int lo_i = max(j, p0);
    // (third case of Eq. 15: a key among the last block's positions is visible to every later row)
    const int hi_i = windowed && !(EQ15 && j >= p.last_lo) ? min(p.L - 1, j + p.w - 1) : p.L - 1;
    const unsigned span = (unsigned)(hi_i - lo_i);
    const bool any = key_ok && hi_i >= lo_i;
#pragma unroll
    for (int s = 0; s < UNITS; ++s) {
      const uint4 rc = rc_s[par][32 * s + lq];  // this lane's row of the unit
      f32x16 sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(split_operand(rc.x, rc.y), ones, zero16, 0, 0, 0);
      f32x16 gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(split_operand(rc.z, rc.w), ones, zero16, 0, 0, 0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(qs, 2 * 32 * s * D + ro.row[kk]), kf[kk], sacc, 0, 0, 0);
        gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_row(gsm, 2 * 32 * s * D + ro.row[kk]), vf[kk], gacc, 0, 0, 0);
      }
      if (masked) {
        const int base = Iq * BLK + 32 * s + 4 * lh;
        if (sub && windowed && Iq > I_hi && (Iq + 1) * BLK <= p.L) {
          // a whole query block J + 2^r' above the window range: visible iff row and key share the mask
          // block within their tiles (no window; a last-block key lies in the last two blocks, whose
          // rows are all inside the window range of their own and the previous block)
          const int jo = j & (BLK - 1);
          const int qb = 32 * s + 4 * lh;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int qio = qb + 8 * (i >> 2) + (i & 3);
            sacc[i] = (((jo ^ qio) >> sub_sh) == 0 && key_ok) ? sacc[i] : kNegInf;
          }
        } else if (sub && windowed) {
          // window range, or (valid, causal and) a power-of-two mask-block distance, or a last-block key
          const unsigned cspan = (unsigned)(p.L - 1 - lo_i);
          const int kmb = j >> sub_sh;
          const bool last = j >= p.last_lo;
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int qi = base + 8 * (i >> 2) + (i & 3);
            const int x = (qi >> sub_sh) - kmb;
            const bool far = key_ok & ((unsigned)(qi - lo_i) <= cspan) & ((x > 0 && (x & (x - 1)) == 0) | last);
            const bool vis = (any & ((unsigned)(qi - lo_i) <= span)) | far;
            sacc[i] = vis ? sacc[i] : kNegInf;
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int qi = base + 8 * (i >> 2) + (i & 3);
            const bool vis = any & ((unsigned)(qi - lo_i) <= span);
            sacc[i] = vis ? sacc[i] : kNegInf;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sacc[i] = __builtin_amdgcn_exp2f(sacc[i]);  // P
        gacc[i] *= sacc[i];                         // dS
      }
      bf16x8 pf[2], dsf[2];
      to_operand(sacc, pf);
      to_operand(gacc, dsf);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          dv[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(gsm, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), pf[t],
                                                           dv[mb], 0, 0, 0);
          dk[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(qs, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), dsf[t],
                                                           dk[mb], 0, 0, 0);
        }
      if (hp) {  // rows with few keys: large P and dS, add the rounding residuals as a second bf16 term
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
            dv[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(gsm, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), pf[t],
                                                             dv[mb], 0, 0, 0);
            dk[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_tr(qs, 2 * (32 * s + 16 * t) * D + ro.tr[mb], 2 * (32 * s + 16 * t) * D + ro.tr8[mb]), dsf[t],
                                                             dk[mb], 0, 0, 0);
          }
      }
    }
  };

  int ent_cur = entry_of(0);
  int ent_nxt = entry_of(min(1, n_all - 1));
  {
    const int I0 = ent_cur & kInvBlockMask;
    const bool win0 = 0 < n_st;
    sg.stage(q_lane, Qs0, I0);
    sg.stage(win0 ? gs_lane : gl_lane, Gs0, I0);
    const uint4 r0 = row_consts(I0, win0);
    if (tid < BLK) rc_s[0][tid] = r0;
  }
  __syncthreads();
  auto step = [&](int t, uint16_t *q_fill, uint16_t *g_fill, const uint16_t *q_cur, const uint16_t *g_cur,
                  int par) __attribute__((always_inline)) {
    uint4 rn = pad_consts;
    const bool more = t + 1 < n_all;
    const int ent_after = entry_of(min(t + 2, n_all - 1));  // consumed at the end of this step
    if (more) {
      const int In = ent_nxt & kInvBlockMask;
      const bool win_n = t + 1 < n_st;
      rn = row_consts(In, win_n);
      sg.stage(q_lane, q_fill, In);
      sg.stage(win_n ? gs_lane : gl_lane, g_fill, In);
    }
    const bool win = t < n_st;
    const int Iq = ent_cur & kInvBlockMask;
    // rows that may see fewer than kFewKeys keys: the first valid rows of a window (or a very
    // short window), or a query block flagged by the inverse list
    const bool hp = win ? (p.w < kFewKeys || Iq * BLK - p0 + 1 < kFewKeys) : (ent_cur >> kInvFewShift) != 0;
    tile_body(q_cur, g_cur, par, Iq, win, hp);
    if (more && tid < BLK) rc_s[par ^ 1][tid] = rn;
    ent_cur = ent_nxt;
    ent_nxt = ent_after;
    __syncthreads();
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Qs1, Gs1, Qs0, Gs0, 0);
    if (t + 1 < n_all) step(t + 1, Qs0, Gs0, Qs1, Gs1, 1);
  }

  // ---- residual passes over the query blocks with few-key rows ----
  // There the probabilities are near one, dV holds single terms P*dO_x of full size and dS
  // projections of dO_x that are small against its norm, so the bf16 rounding of dO_x itself
  // would show.  Everything above is linear in dO_x: the tile is simply walked a second time
  // with the residual dO_x - bf16(dO_x) in place of dO_x and residual.o_x in place of c_x.  The
  // residual tile is rebuilt in LDS from dO, alpha, dz and the gate weights exactly as the
  // per-row pass formed dO_x.  (Rare: the first blocks of a row, or top-k below three.)
  auto residual_pass = [&](int Iq, bool windowed) __attribute__((always_inline)) {
    sg.stage(q_lane, Qs0, Iq);
    {
      // thread -> (row, half of d): 32 residuals each, written as four swizzled 16-byte chunks
      const int r = tid >> 1, hf = tid & 1;
      const int i = Iq * BLK + r;
      const bool in = i < p.L;
      const size_t ro = head + (size_t)min(i, p.L - 1) * D + 32 * hf;
      const float4 st = rowstat[lbase + min(i, p.L - 1)];
      const float ax = windowed ? 1.0f - st.x : st.x;
      const float *wrow = gate_w + (size_t)(bh % p.H) * 2 * D + (windowed ? D : 0) + 32 * hf;
      const float *orow = (windowed ? o_st : o_lt) + ro;
      float corr = 0.0f;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(dO + ro + 8 * c);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        uint32_t out[4];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float g = (e & 1) ? bf_hi(w[e >> 1]) : bf_lo(w[e >> 1]);
          const float full = fmaf(ax, g, st.y * wrow[8 * c + e]);
          const uint16_t lo = in ? f32_to_bf16(full - bf16_to_f32(f32_to_bf16(full))) : (uint16_t)0;
          corr = fmaf(bf16_to_f32(lo), orow[8 * c + e], corr);
          if (e & 1) out[e >> 1] |= (uint32_t)lo << 16; else out[e >> 1] = lo;
        }
        const int chunk = (4 * hf + c) ^ swz(r);
        *reinterpret_cast<uint4 *>(Gs0 + r * D + chunk * 8) = make_uint4(out[0], out[1], out[2], out[3]);
      }
      corr += __shfl_xor(corr, 1);
      if (hf == 0) {
        const uint4 base = in ? (windowed ? rowI_st : rowI_lt)[lbase + i] : pad_consts;
        const uint2 k = split3(-corr);
        rc_s[0][r] = make_uint4(base.x, base.y, k.x, k.y);
      }
    }
    __syncthreads();  // (waits for the staged Q rows of every wavefront as well)
    tile_body(Qs0, Gs0, 0, Iq, windowed, false);
    __syncthreads();
  };
  if (p.w < kFewKeys || J * BLK - p0 + 1 < kFewKeys) {  // the window part: a prefix of the walk
#pragma unroll 1
    for (int t = 0; t < n_st; ++t) {
      const int Iq = entry_of(t);
      if (!(p.w < kFewKeys || Iq * BLK - p0 + 1 < kFewKeys)) break;
      residual_pass(Iq, true);
    }
  }
#pragma unroll 1
  for (int e = 0; e < n_lt; ++e) {  // flagged entries of the inverse list
    const int ent = __builtin_amdgcn_readfirstlane(my_items[e]);
    if ((ent >> kInvFewShift) != 0) residual_pass(ent & kInvBlockMask, false);
  }

  {  // (every wavefront is past the last barrier of the walk: the staging rows are free)
    const int row0 = J * BLK + 32 * wv;
    store_rows_bf16(dK + head + (size_t)row0 * D, p.L - row0, Qs0 + wv * 32 * D, dk, p.scale, key_ok, p, true, row0);
    store_rows_bf16(dV + head + (size_t)row0 * D, p.L - row0, Gs0 + wv * 32 * D, dv, 1.0f, key_ok, p);
  }
}

#define BWD_LDS_TILES(BLK)                                                   \
  __shared__ __attribute__((aligned(1024))) uint16_t lds_t0[(BLK) * D];      \
  __shared__ __attribute__((aligned(1024))) uint16_t lds_t1[(BLK) * D];      \
  __shared__ __attribute__((aligned(1024))) uint16_t lds_t2[(BLK) * D];      \
  __shared__ __attribute__((aligned(1024))) uint16_t lds_t3[(BLK) * D]

#define BWD_DQ_PARAMS                                                                                              \
  const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,                  \
      const int *__restrict__ valid_len, const int *__restrict__ sel, const uint16_t *__restrict__ g_lt,           \
      const uint16_t *__restrict__ g_st, const uint4 *__restrict__ rowI_lt, const uint4 *__restrict__ rowI_st,     \
      const uint16_t *__restrict__ dO, const float4 *__restrict__ rowstat, const float *__restrict__ gate_w,       \
      const float *__restrict__ o_lt, const float *__restrict__ o_st, uint16_t *__restrict__ dQ
#define BWD_DQ_ARGS Q, K, V, valid_len, sel, g_lt, g_st, rowI_lt, rowI_st, dO, rowstat, gate_w, o_lt, o_st, dQ
#define BWD_DKV_ARGS Q, K, V, valid_len, g_lt, g_st, rowI_lt, rowI_st, offs, items, dO, rowstat, gate_w, o_lt, o_st, dK, dV

template <int BLK, bool EQ15, bool SUB>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_dq_mfma_kernel(BWD_DQ_PARAMS, KParams p)
{
  BWD_LDS_TILES(BLK);
  bwd_dq_body<BLK, EQ15, SUB>(BWD_DQ_ARGS, p, blockIdx.x, lds_t0, lds_t1, lds_t2, lds_t3);
}

template <int BLK, bool EQ15, bool SUB>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_dkv_mfma_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int *__restrict__ valid_len, const uint16_t *__restrict__ g_lt, const uint16_t *__restrict__ g_st,
    const uint4 *__restrict__ rowI_lt, const uint4 *__restrict__ rowI_st, const int *__restrict__ offs,
    const int *__restrict__ items, const uint16_t *__restrict__ dO, const float4 *__restrict__ rowstat,
    const float *__restrict__ gate_w, const float *__restrict__ o_lt, const float *__restrict__ o_st,
    uint16_t *__restrict__ dK, uint16_t *__restrict__ dV, KParams p)
{
  BWD_LDS_TILES(BLK);
  __shared__ __attribute__((aligned(16))) uint4 rc_s[2][BLK];
  bwd_dkv_body<BLK, EQ15, SUB>(BWD_DKV_ARGS, p, blockIdx.x, lds_t0, lds_t1, lds_t2, lds_t3, rc_s);
}

// dQ and dK/dV in ONE launch (the full backward call): the first B*H*NB workgroups take the key blocks, the
// rest the query blocks.  The two kernels need the same workgroup shape, the same two wavefronts per SIMD and
// nearly the same LDS, so nothing is lost by the union, and the short dQ workgroups fill the slots that the
// tail of the skewed dK/dV walks leaves idle (and one launch gap goes).
template <int BLK, bool EQ15, bool SUB>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_both_mfma_kernel(
    BWD_DQ_PARAMS, const int *__restrict__ offs, const int *__restrict__ items, uint16_t *__restrict__ dK,
    uint16_t *__restrict__ dV, KParams p)
{
  BWD_LDS_TILES(BLK);  // the four staging tiles serve either role
  __shared__ __attribute__((aligned(16))) uint4 rc_s[2][BLK];
  const unsigned n = (unsigned)(p.B * p.H * p.NB);
  if (blockIdx.x < n) bwd_dkv_body<BLK, EQ15, SUB>(BWD_DKV_ARGS, p, blockIdx.x, lds_t0, lds_t1, lds_t2, lds_t3, rc_s);
  else bwd_dq_body<BLK, EQ15, SUB>(BWD_DQ_ARGS, p, blockIdx.x - n, lds_t0, lds_t1, lds_t2, lds_t3);
}

bool bwd_mfma_supported(const KParams &p, int dtype)
{
  return dtype == 1 && p.d == 64 && (p.b == 32 || p.b == 64) && !p.bidir &&
         (p.sblk == 0 || (is_pow2(p.sblk) && p.sblk <= p.b));
}

void launch_bwd_mfma(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st)
{
  const bool do_dq = stages & kBwdStageDQ, do_dkv = stages & kBwdStageDKV;
  const unsigned grid = (unsigned)(p.B * p.H * p.NB);
  auto u16 = [](const void *x) { return reinterpret_cast<const uint16_t *>(x); };
  auto go_dq = [&](auto kernel, unsigned threads) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, st, u16(a.Q), u16(a.K), u16(a.V), a.valid_len, a.sel,
                       w.g_lt, w.g_st, w.rowI_lt, w.rowI_st, u16(a.dO), w.rowstat, a.gate_w, (const float *)a.o_lt,
                       (const float *)a.o_st, (uint16_t *)a.dQ, p);
  };
  auto go_dkv = [&](auto kernel, unsigned threads) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, st, u16(a.Q), u16(a.K), u16(a.V), a.valid_len, w.g_lt,
                       w.g_st, w.rowI_lt, w.rowI_st, w.offs, w.items, u16(a.dO), w.rowstat, a.gate_w,
                       (const float *)a.o_lt, (const float *)a.o_st, (uint16_t *)a.dK, (uint16_t *)a.dV, p);
  };
  const bool eq15 = p.sblk != 0;
  const bool sub = eq15 && p.sblk < p.b;  // mask block smaller than the tile
  if (do_dq && do_dkv && 2ull * grid <= 0x7FFFFFFFull) {
    auto go = [&](auto kernel, unsigned threads) {
      hipLaunchKernelGGL(kernel, dim3(2 * grid), dim3(threads), 0, st, u16(a.Q), u16(a.K), u16(a.V), a.valid_len, a.sel,
                         w.g_lt, w.g_st, w.rowI_lt, w.rowI_st, u16(a.dO), w.rowstat, a.gate_w, (const float *)a.o_lt,
                         (const float *)a.o_st, (uint16_t *)a.dQ, w.offs, w.items, (uint16_t *)a.dK, (uint16_t *)a.dV, p);
    };
    if (p.b == 32) {
      if (sub) go(bwd_both_mfma_kernel<32, true, true>, 64);
      else if (eq15) go(bwd_both_mfma_kernel<32, true, false>, 64);
      else go(bwd_both_mfma_kernel<32, false, false>, 64);
    } else {
      if (sub) go(bwd_both_mfma_kernel<64, true, true>, 128);
      else if (eq15) go(bwd_both_mfma_kernel<64, true, false>, 128);
      else go(bwd_both_mfma_kernel<64, false, false>, 128);
    }
    return;
  }
  if (p.b == 32) {
    if (do_dq) {
      if (sub) go_dq(bwd_dq_mfma_kernel<32, true, true>, 64);
      else if (eq15) go_dq(bwd_dq_mfma_kernel<32, true, false>, 64);
      else go_dq(bwd_dq_mfma_kernel<32, false, false>, 64);
      if (launch_failed()) return;
    }
    if (do_dkv) {
      if (sub) go_dkv(bwd_dkv_mfma_kernel<32, true, true>, 64);
      else if (eq15) go_dkv(bwd_dkv_mfma_kernel<32, true, false>, 64);
      else go_dkv(bwd_dkv_mfma_kernel<32, false, false>, 64);
    }
  } else {
    if (do_dq) {
      if (sub) go_dq(bwd_dq_mfma_kernel<64, true, true>, 128);
      else if (eq15) go_dq(bwd_dq_mfma_kernel<64, true, false>, 128);
      else go_dq(bwd_dq_mfma_kernel<64, false, false>, 128);
      if (launch_failed()) return;
    }
    if (do_dkv) {
      if (sub) go_dkv(bwd_dkv_mfma_kernel<64, true, true>, 128);
      else if (eq15) go_dkv(bwd_dkv_mfma_kernel<64, true, false>, 128);
      else go_dkv(bwd_dkv_mfma_kernel<64, false, false>, 128);
    }
  }
}

}  // namespace blossom

// Fused forward on the matrix cores for bf16, d = 64, block size 32 or 64 (Eq. 1 under the two
// branch masks, Eq. 16-19), plus the same-style dense causal comparison.
//
// Work split: one workgroup per (row, head, query block), BLK/32 wavefronts.  Every wavefront
// works on ALL query rows of the block but only on "its" 32 key rows of every K/V tile (keys
// 32*wv .. 32*wv+31 of the block): it stages those rows itself with direct global->LDS loads
// (16 bytes per lane, whole 128-byte rows per 8 lanes, XOR-swizzled so that the operand reads
// are bank-conflict free), and nobody else reads them.  The tile loop therefore has no
// workgroup barrier at all; a wavefront only waits for its own loads.  Each K fragment read
// from LDS serves all query groups, each V fragment too.  At the end of a branch the wavefronts
// hold partial (reference, row sum, output) triples over disjoint key subsets; they are merged
// through LDS once per branch, after which wavefront wv owns the finished rows 32*wv .. +31.
//
// Per tile and 32-query group a wavefront computes S^T = K Q^T with four
// v_mfma_f32_32x32x16_bf16 (keys are the M dimension, so every lane owns ONE query column and
// 16 of its logits: row maximum and row sum are in-lane reductions plus one exchange with
// lane^32), applies the online softmax in fp32, and feeds P^T straight from the accumulator
// registers (converted to bf16) as the B operand of O^T += V^T P^T (four more MFMAs).  The key
// order inside a contraction slab is whatever the accumulator layout dictates; V^T is read
// from LDS with the transposing ds_read_b64_tr_b16 in exactly that order, so P never moves
// between lanes.
//
// Softmax bookkeeping: Q is pre-multiplied by scale*log2(e) (rounded to bf16 once), and the
// logits of a tile are started by one extra matrix instruction that broadcasts minus the row's
// current reference m_ref (an exact three-term bf16 split), so the MFMA result is directly the
// exponent s*c - m_ref and each probability costs one v_exp_f32, with no per-element VALU
// initialisation.  The common tile takes its exponentials speculatively against the current
// references and is accepted when every lane's probabilities sum to at most 2^12; only a
// branch's first visible key, or a maximum that ran more than 2^8 above the reference, sends
// the tile through the slow path (row maxima, shift of the tile's exponents, the running sum
// and the output accumulators, exponentials again).  Row sums are plain fp32 adds: the packed
// dot-product instructions execute on the matrix pipeline and would stall the MFMAs.
//
// The walk: the short-term branch first (window blocks by arithmetic; with the full mask of
// Eq. 15, compile-time variant EQ15, also the blocks 2^r before the query block: whole tiles when
// the mask block is BLK, masked element by element in the variant SUB for smaller power-of-two
// mask blocks), then the long-term branch, whose
// block ids come from one scalar load per tile out of the selection row, issued a tile ahead.
// Outputs leave through the wavefront's staging rows so that every store covers whole rows.
#include "launch.h"
#include "mfma_common.h"

namespace blossom {

using namespace mfma;

namespace {

constexpr float kRaise = 8.0f;  // log2 units by which the maximum must grow before it is raised
constexpr int kFewKeys = 32;    // rows seeing fewer keys than this get two-term bf16 probabilities
constexpr float kSumLimit = 4096.0f;  // a lane's 16 probabilities of a tile may sum to this (16 * 2^kRaise)

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding and
// leaves the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4,
// lgkmcnt 11:8).
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

}  // namespace

// EQ15: the short-term mask is all of Eq. 15 with mask block BLK, or (SUB) a power of two below it
// (compile-time, so that the plain causal window compiles to exactly the code it had without it)
template <int BLK, bool EQ15, bool SUB>
__global__ __launch_bounds__(BLK * 2) __attribute__((amdgpu_waves_per_eu(BLK == 32 ? 3 : 2, BLK == 32 ? 3 : 2))) void fwd_mfma_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int *__restrict__ valid_len, const int *__restrict__ sel, const float *__restrict__ gate_w,
    const float *__restrict__ gate_b, uint16_t *__restrict__ O, float *__restrict__ o_lt_out,
    float *__restrict__ o_st_out, float *__restrict__ lse_lt_out, float *__restrict__ lse_st_out, int dense,
    KParams p)
{
  constexpr int NQ = BLK / 32;   // 32-query groups per wavefront == wavefronts per workgroup
  constexpr int TILE = BLK * D;  // bf16 elements of one staged tile (rows of 128 bytes, swizzled)
  constexpr int HALF = 32 * D;   // elements of the 32 rows one wavefront stages and reads
  // Four separate arrays (not one indexed by parity): the compiler can then prove that a
  // prefetch in flight into one buffer does not alias the operand reads of another, and does
  // not wait for the prefetch before those reads.
  __shared__ __attribute__((aligned(1024))) uint16_t Ks0[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Ks1[TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs0[TILE];
  // The 32-row kernel (one wavefront per workgroup, short tiles) is bound by latency, so it trades
  // the second V buffer for a third wavefront per SIMD (12.5 KB of LDS and 168 registers per
  // workgroup): a tile's V is requested at the start of its own step, ahead of the next K tile,
  // and waited for after the QK products.
  constexpr bool V1 = BLK == 32;
  __shared__ __attribute__((aligned(1024))) uint16_t Vs1[V1 ? 8 : TILE];
  __shared__ float gate_s[2 * D];     // this head's gate weights, fetched at the start, used at the very end
  __shared__ float xch_s[NQ][2][64];  // branch merge: reference and partial row sum handed to the partner

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // readfirstlane tells the compiler the wavefront index is uniform, so every branch that
  // depends on it is a scalar branch: matrix instructions ignore EXEC and must never sit in a
  // region that is merely masked off.
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31;  // query column (and key row of the K operand, d row of the V^T operand)
  const int lh = lane >> 5;  // which half of each 16-wide contraction slab
  const unsigned vid = xcd_remap(blockIdx.x, (unsigned)(p.B * p.H * p.nq));
  const int bh = (int)(vid / p.nq);
  const int I = p.NB - 1 - (int)(vid % p.nq);
  const int h = bh % p.H;
  const size_t head = (size_t)bh * p.L * D;
  // Local query group g covers rows I*BLK + 32*(g ^ wv) + lq: group 0 is always the one this
  // wavefront finishes and stores, group 1 the one it hands to its partner.
  int qbase[NQ], iq[NQ];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    qbase[g] = I * BLK + 32 * (g ^ wv);
    iq[g] = qbase[g] + lq;
  }

  // ---- everything the prologue needs from memory is requested before anything is waited for ----
  const int n_raw = valid_len[bh / p.H];
  uint4 qraw[NQ][4];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    const uint16_t *qrow = Q + head + (size_t)min(iq[g], p.L - 1) * D;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qraw[g][kk] = *reinterpret_cast<const uint4 *>(qrow + 16 * kk + 8 * lh);
  }
  const int *my_sel = dense ? nullptr : sel + ((size_t)bh * p.NB + I) * p.k;
  const int sel0 = (!dense && lane < p.k) ? my_sel[lane] : -1;  // first 64 entries of the selection row
  constexpr int GATE_PER = 2 * D / (2 * BLK);                    // gate weights fetched per thread
  float gate_mine[GATE_PER];
#pragma unroll
  for (int c = 0; c < GATE_PER; ++c) gate_mine[c] = dense ? 0.0f : gate_w[(size_t)h * 2 * D + c * 2 * BLK + tid];

  const int n = clamp_len(n_raw, p.L);
  const int p0 = p.L - n;
  bool q_ok[NQ];
#pragma unroll
  for (int g = 0; g < NQ; ++g) q_ok[g] = iq[g] < p.L && iq[g] >= p0;

  if (min((I + 1) * BLK, p.L) <= p0) {  // no valid query in the block: zero outputs (this wavefront's 32 rows)
    zero_rows(O + head, qbase[0], 32, p.L, lane);
    if (o_lt_out) {
      zero_rows(o_lt_out + head, qbase[0], 32, p.L, lane);
      zero_rows(o_st_out + head, qbase[0], 32, p.L, lane);
    }
    if (iq[0] < p.L && lh == 0) {
      if (lse_lt_out) lse_lt_out[(size_t)bh * p.L + iq[0]] = 0.0f;
      if (lse_st_out) lse_st_out[(size_t)bh * p.L + iq[0]] = 0.0f;
    }
    return;
  }

  // window blocks J_lo..I come first in the walk; they depend on the valid length only
  const int J_first = p0 / BLK;
  // With the full short-term mask (Eq. 15) the blocks I - 2^r below the window range follow:
  // r = r0 .. r0 + n_pow - 1.  The mask block is BLK or a power of two below it (`sub`): then the
  // mask-block distances 2^r below one tile reach into block I - 1, which joins the window range,
  // the larger ones land on the same blocks I - 2^r' (at the row's own offset), and every
  // short-term tile is masked element by element with the three cases of Eq. 15.
  constexpr bool sub = EQ15 && SUB;  // (compile-time: the mask block = BLK variant keeps its code and registers)
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
      const int d_win = I - J_lo;                                       // largest block distance inside the window range
      r0 = d_win == 0 ? 0 : 32 - __builtin_clz((unsigned)d_win);        // smallest r with 2^r > d_win
      const int r_max = 31 - __builtin_clz((unsigned)(I - J_first));  // largest r with I - 2^r >= J_first
      n_st += max(0, r_max - r0 + 1);
    }
  }

  // ---- staging: each wavefront moves its 32 rows (4 x 1 KB) of K and of V per tile ----
  // LDS position of 16-byte chunk c of row r:  r*128 + ((c ^ swz(r)) * 16),
  //   swzK(r) = (r >> 1) & 7 for the row-per-lane 16-byte reads.  Measured on gfx950: the LDS serves
  //             16 lanes x 16 bytes per cycle over 64 banks, rows of 128 bytes alternate between the
  //             two bank halves, and a cycle's lanes run over bits 1-3 of the lane index (bit 4
  //             tied to them, bit 0 free): positions must be distinct over row bits 1-3.
  //   swzV(r) = 2*(r & 3) (4 rows x two chunk columns = 8 distinct positions for the transposing reads)
  // A tile's rows are contiguous in memory, and the LDS copy keeps the 128-byte row pitch, so
  // one uniform base (SGPRs) + one per-lane byte offset + the same immediate for the global
  // and the LDS side addresses all four 8-row slices.
  const char *Kh = reinterpret_cast<const char *>(K + head);
  const char *Vh = reinterpret_cast<const char *>(V + head);
  const int ld_row = 32 * wv + (lane >> 3);  // + 8*u
  // rows 8u .. 8u+7 of a slice: swzK = (lane >> 4) | ((u & 1) << 2), so odd slices use k_lane ^ 64
  const unsigned k_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (lane >> 4)) * 8) * 2u;            // bytes
  const unsigned v_lane = (unsigned)(ld_row * D + ((lane & 7) ^ (2 * ((lane >> 3) & 3))) * 8) * 2u;  // bytes
  const bool ragged = p.L % BLK != 0;
  auto stage = [&](const char *src_head, unsigned lane_off, unsigned odd_xor, uint16_t *dst_tile, int J) __attribute__((always_inline)) {
    const char *src = src_head + (size_t)max(J, 0) * (TILE * 2);  // uniform (block -1: any block will do, all of it is masked)
    lds_void *dst = (lds_void *)(dst_tile + 32 * wv * D);
    if (!ragged || J != p.NB - 1) {
      const unsigned lane_odd = lane_off ^ odd_xor;  // odd 8-row slices (K only: their swizzle differs)
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 1024, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_off), dst, 16, 2048, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(src + lane_odd), dst, 16, 3072, 0);
    } else {  // last, partial block: rows past the end are clamped (they are causally masked anyway)
      // (the empty asm hides that J is a constant here: the clamped per-lane offsets would
      // otherwise be computed ahead of the loop and held in registers throughout)
      asm volatile("" : "+s"(J));
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int over = max(0, J * BLK + ld_row + 8 * u - (p.L - 1));
        const unsigned off = ((u & 1) ? lane_off ^ odd_xor : lane_off) + (unsigned)((8 * u - over) * D * 2);
        __builtin_amdgcn_global_load_lds((glb_void *)(src + off), (lds_void *)(dst_tile + (32 * wv + 8 * u) * D), 16, 0, 0);
      }
    }
  };

  // the first tile is on its way while the rest of the prologue runs
  const int first_J = dense ? J_first : J_lo;
  stage(Kh, k_lane, 64u, Ks0, first_J);
  if (!V1) stage(Vh, v_lane, 0u, Vs0, first_J);

  // Q^T operand: lane (query lq, half lh) holds c*Q[iq][16*kk + 8*lh .. +7] for the 4 slabs kk,
  // c = scale*log2(e), rounded to bf16: the matrix cores then produce base-2 exponents directly.
  const float c2 = p.scale * kLog2e;
  bf16x8 qf[NQ][4];
#pragma unroll
  for (int g = 0; g < NQ; ++g)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const uint32_t w[4] = {qraw[g][kk].x, qraw[g][kk].y, qraw[g][kk].z, qraw[g][kk].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        qf[g][kk][2 * e] = (__bf16)(bf_lo(w[e]) * c2);
        qf[g][kk][2 * e + 1] = (__bf16)(bf_hi(w[e]) * c2);
      }
    }
  if (!dense)
#pragma unroll
    for (int c = 0; c < GATE_PER; ++c) gate_s[c * 2 * BLK + tid] = gate_mine[c];

  // ---- tile list: window blocks J_lo..I, then the selection list up to its last valid entry ----
  // Every wavefront reads the whole selection row with one vector load per 64 entries and
  // derives the counts from ballots (no chain of dependent scalar loads).  The walk itself
  // fetches one entry per tile with a scalar load (see tile_raw): those do not touch the
  // vector-memory counter, which tracks the tile prefetches in flight.
  int n_all;
  bool lt_few = true;  // the selected past blocks hold fewer than kFewKeys valid keys
  if (dense) {
    n_all = I - J_first + 1;
  } else {
    // Entries outside [0, NB) are skipped wherever they stand: the walk runs up to the last valid
    // entry, and an invalid one in between costs one tile whose keys are all masked (block id -1).
    int n_lt = 0;
    for (int e0 = 0; e0 < p.k; e0 += 64) {
      const int e = e0 + lane;
      const int J = e0 == 0 ? sel0 : (e < p.k ? my_sel[e] : -1);
      const bool ok = J >= 0 && J < p.NB;
      const unsigned long long okm = __ballot(ok);
      if (okm != 0ull) n_lt = e0 + 64 - __builtin_clzll(okm);
      // a full earlier block already brings a whole block of keys; only a partial first block may not
      const int vcount = min((J + 1) * BLK, p.L) - max(J * BLK, p0);
      if (__ballot(ok && J < I && vcount >= kFewKeys) != 0ull) lt_few = false;
    }
    n_all = n_st + n_lt;
  }
  __syncthreads();
  // Block id of tile t: window blocks by arithmetic, selected blocks by a scalar load from the
  // selection row (uniform address), issued a whole tile before its value is needed.
  auto tile_raw = [&](int t) -> int {
    if (dense) return J_first + t;
    const int e = __builtin_amdgcn_readfirstlane(t - n_st);
    typedef const int __attribute__((address_space(4))) *const_int_ptr;  // read-only: loads become scalar
    if (e >= 0) return ((const_int_ptr)my_sel)[e];  // raw: may be outside [0, NB), see list_entry
    if (!EQ15) return J_lo + t;
    return t < n_win ? J_lo + t : I - (1 << (r0 + t - n_win));
  };

  // a raw tile-list value when it is consumed (a whole tile after its scalar load was issued): entries
  // outside [0, NB) become -1, a tile whose keys are all masked
  auto list_entry = [&](int raw) -> int {
    const int J = __builtin_amdgcn_readfirstlane(raw);
    return (unsigned)J < (unsigned)p.NB ? J : -1;
  };

  // ---- per-lane LDS read offsets (elements) inside this wavefront's 32 rows ----
  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) koff[kk] = wv * HALF + lq * D + (((2 * kk + lh) ^ ((lq >> 1) & 7)) * 8);
  const int r16 = lane & 15;
  int voff[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
    voff[mb] = wv * HALF + (4 * lh + (r16 >> 2)) * D +
               (((4 * mb + 2 * ((lane >> 4) & 1) + ((r16 & 3) >> 1)) ^ (2 * (r16 >> 2))) * 8) + 4 * (r16 & 1);

  // Per-row softmax state of each query group.  m_ref: reference exponent (log2 units) the
  // accumulators are relative to; fresh: no visible key met yet in this branch; l_run: this
  // lane's part of the row sum.  Rows that are padding never become valid: they are not
  // "fresh" either, so they never ask for the slow path below (their outputs are zeroed).
  f32x16 oacc[NQ][2];
  float m_ref[NQ], l_run[NQ];
  bool fresh[NQ];
  // -m_ref as an operand: the logits of a tile are started by one extra matrix instruction
  // ones[key][0..2] x (hi, mid, lo of -m_ref)[0..2][query], a three-term bf16 split that
  // represents the fp32 value exactly, so no per-element VALU initialisation is needed.
  bf16x8 mneg[NQ];
  bf16x8 ones_k;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones_k[e] = (__bf16)((lh == 0 && e < 3) ? 1.0f : 0.0f);
  auto set_ref = [&](int g, float m) __attribute__((always_inline)) {
    m_ref[g] = m;
    const float x = -m;
    const __bf16 hi = (__bf16)x;
    const float r1 = x - (float)hi;
    const __bf16 mid = (__bf16)r1;
    const __bf16 lo = (__bf16)(r1 - (float)mid);
    const __bf16 zero = (__bf16)0.0f;
    mneg[g] = bf16x8{lh == 0 ? hi : zero, lh == 0 ? mid : zero, lh == 0 ? lo : zero, zero, zero, zero, zero, zero};
  };
#pragma unroll
  for (int g = 0; g < NQ; ++g) set_ref(g, 0.0f);
  auto reset = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      fresh[g] = q_ok[g];
      l_run[g] = 0.0f;
#pragma unroll
      for (int i = 0; i < 16; ++i) { oacc[g][0][i] = 0.0f; oacc[g][1][i] = 0.0f; }
    }
  };

  // Rows that see only a few keys have large probabilities, and rounding those to bf16 would
  // leave a relative error of 2^-9 in the saved branch outputs, which backward amplifies
  // through D = dO_x.o_x.  Blocks that may hold such rows (fewer than kFewKeys keys) feed P to
  // the matrix cores as a two-term bf16 sum (hi + lo); everyone else uses one term.
  int hp_st, hp_lt;  // uniform
  if (dense) {
    hp_st = 0;
    hp_lt = I * BLK - p0 + 1 < kFewKeys;
  } else {
    hp_st = p.w < kFewKeys || I * BLK - p0 + 1 < kFewKeys;
    hp_lt = __builtin_amdgcn_readfirstlane((int)lt_few);
  }

  // ---- per-tile pieces ----
  // visible <=> lo <= key <= iq with lo = max(p0, iq - w + 1); per lane this is one range test
  // on the element's compile-time key offset
  auto mask = [&](int J, bool windowed, int g, f32x16 &s) __attribute__((always_inline)) {
    // (The query row is rebuilt from the lane id inside a volatile asm: everything derived
    // below would otherwise be loop invariant, get hoisted, and sit in registers or spill
    // slots across the whole walk.)
    int ql;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ql));
    const int q = qbase[g] + (ql & 31);
    const int lh = ql >> 5;
    asm volatile("" : "+s"(J));
    int wlo = q - p.w + 1;
    if (EQ15 && q >= p.last_lo) wlo = min(wlo, p.last_lo);  // third case of Eq. 15: the last block is visible to its own rows
    const int lo = windowed ? max(p0, wlo) : p0;
    const int base = J * BLK + 32 * wv + 4 * lh;
    const unsigned span = (unsigned)(q - lo);  // wraps to huge when q < lo: handled by `any`
    const bool any = q >= lo;
    if (EQ15 && sub && windowed && J < J_lo && J * BLK >= p0) {
      // A block I - 2^r' below the window range, all of it valid: no key of it lies in a window or in
      // the last block, and a mask-block distance 2^r' * (BLK / blk) + delta with |delta| < BLK / blk <=
      // half of it is a power of two only for delta = 0: row and key share the mask block within their tiles.
      const int qo = q & (BLK - 1);
      const int kb = 32 * wv + 4 * lh;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int ko = kb + 8 * (i >> 2) + (i & 3);
        s[i] = (((qo ^ ko) >> sub_sh) == 0 && q >= p0) ? s[i] : kNegInf;
      }
      return;
    }
    if (EQ15 && sub && windowed) {
      // window range as above, or (valid, causal and) a power-of-two mask-block distance, or a last-block key
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
    // the other half of the wavefront's keys for this query lives in lane^32
    const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  };
  // Slow path of the reference bookkeeping: moves the reference of group g to the tile maximum
  // where a row meets its first visible key or where the maximum ran away upwards, and shifts
  // the tile's exponents, the running sum and the output accumulators accordingly.
  auto move_ref = [&](int g, f32x16 &s) __attribute__((always_inline)) {
    const float mx = row_max(s);
    const bool upd = fresh[g] ? mx != kNegInf : mx > kRaise;
    const float dlt = upd ? mx : 0.0f;
    const float alpha = (upd && !fresh[g]) ? __builtin_amdgcn_exp2f(-dlt) : 1.0f;
    l_run[g] *= alpha;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[g][0][i] *= alpha; oacc[g][1][i] *= alpha; }
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] -= dlt;
    set_ref(g, m_ref[g] + dlt);
    fresh[g] = fresh[g] && !upd;
  };

  // exponentials of one group: pf <- bf16(2^s), returns this lane's sum of the probabilities.
  // (Plain fp32 adds: the packed dot-product instructions would do the bf16 sum in one step,
  // but they execute on the matrix pipeline and stall the MFMAs of every wavefront of the SIMD.)
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
  // second bf16 term of P (what the first term's rounding lost); the row sum already holds it
  auto expo_lo = [&](const f32x16 &s, const bf16x8 (&pf)[2], bf16x8 (&pl)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      pl[i >> 3][i & 7] = (__bf16)(__builtin_amdgcn_exp2f(s[i]) - (float)pf[i >> 3][i & 7]);
  };
  // V^T operands of the wavefront's 32 keys: [t][mb], keys in accumulator order
  auto load_v = [&](const uint16_t *vs, bf16x8 (&vf)[2][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const uint16_t *a0 = vs + 16 * t * D + voff[mb];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a0 + 8 * D));
        vf[t][mb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
  };
  auto pv = [&](int g, const bf16x8 (&vf)[2][2], const bf16x8 (&pf)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        oacc[g][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][mb], pf[t], oacc[g][mb], 0, 0, 0);
  };

  // One tile (this wavefront's 32 keys of block J against every query group).
  //
  // The common case costs no bookkeeping beyond the exponentials: they are taken against the
  // current references, and the tile is accepted if every lane's sum of probabilities stays
  // below 2^12 (so no probability can exceed it) and no row is still waiting for its first
  // key.  Otherwise the slow path finds the row maxima, moves the references and takes the
  // exponentials again; it raises a reference whenever a probability would exceed 2^kRaise,
  // which also guarantees that the retaken tile passes.
  auto tile = [&](const uint16_t *ks, const uint16_t *vs, int J, bool short_term, bool last) __attribute__((always_inline)) {
    const bool hp = (short_term ? hp_st : hp_lt) != 0;
    // band-masked by the window, unless Eq. 15 shows the whole block (power-of-two block distance)
    const bool windowed = short_term && !(EQ15 && !sub && is_pow2(I - J));
    // The empty asm makes the read offsets look freshly computed: buffer base + offset is then
    // formed next to each read, where it folds into the instruction's immediate, instead of
    // being kept in one register per (buffer, fragment) across the whole loop.
    asm volatile("" : "+v"(koff[0]), "+v"(koff[1]), "+v"(koff[2]), "+v"(koff[3]), "+v"(voff[0]), "+v"(voff[1]));
    // block-level visibility of the 32 keys for the 32 queries of each group (uniform): tiles
    // whose keys every query sees skip the mask arithmetic
    const int k_lo = J * BLK + 32 * wv, k_hi = k_lo + 31;
    bool full[NQ], all_full = true;
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      const int q_lo = qbase[g], q_hi = qbase[g] + 31;
      full[g] = k_hi <= q_lo && k_lo >= p0 && (!windowed || k_lo >= q_hi - p.w + 1);
      all_full = all_full && full[g];
    }
    f32x16 s[NQ];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < NQ; ++g) s[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones_k, mneg[g], zero16, 0, 0, 0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {  // each K fragment serves every query group
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks + koff[kk]);
#pragma unroll
      for (int g = 0; g < NQ; ++g) s[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[g][kk], s[g], 0, 0, 0);
    }
    if (!all_full) {
#pragma unroll
      for (int g = 0; g < NQ; ++g)
        if (!full[g]) mask(J, windowed, g, s[g]);
    }
    bf16x8 vf[2][2];
    if (V1) {  // this tile's V (4 loads) was requested ahead of the next K tile (4 loads, absent after the last tile)
      if (last) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(4));
    }
    load_v(vs, vf);
    bf16x8 pf[NQ][2];
#pragma unroll
    for (int g = 0; g < NQ; ++g) {  // the P V products of one group run under the exponentials of the next
      float tsum = expo(s[g], pf[g]);
      if (__any(fresh[g] || !(tsum <= kSumLimit))) {
        move_ref(g, s[g]);
        tsum = expo(s[g], pf[g]);
      }
      l_run[g] += tsum;
      pv(g, vf, pf[g]);
    }
    if (hp) {
#pragma unroll
      for (int g = 0; g < NQ; ++g) {
        bf16x8 pl[2];
        expo_lo(s[g], pf[g], pl);
        pv(g, vf, pl);
      }
    }
  };

  // Closes a branch.  With two wavefronts each holds, for every query, a partial result over
  // its own key rows; the partial for the partner's queries (group 1) goes through LDS (staging
  // rows kx/vx of this wavefront, free at this point), the partner's partial for this
  // wavefront's queries comes back the same way, and both are brought to a common reference.
  // Leaves the normalised output of group 0 in oacc[0] and returns its lse (natural log).
  auto close_branch = [&](uint16_t *kx, uint16_t *vx) __attribute__((always_inline)) -> float {
    if constexpr (NQ == 2) {
      float *mine_a = reinterpret_cast<float *>(kx + wv * HALF);  // 16 registers x 64 lanes each
      float *mine_b = reinterpret_cast<float *>(vx + wv * HALF);
      const float *part_a = reinterpret_cast<const float *>(kx + (wv ^ 1) * HALF);
      const float *part_b = reinterpret_cast<const float *>(vx + (wv ^ 1) * HALF);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        mine_a[i * 64 + lane] = oacc[NQ - 1][0][i];
        mine_b[i * 64 + lane] = oacc[NQ - 1][1][i];
      }
      xch_s[wv][0][lane] = fresh[NQ - 1] ? kNegInf : m_ref[NQ - 1];
      xch_s[wv][1][lane] = l_run[NQ - 1];
      __syncthreads();
      const float m_b = xch_s[wv ^ 1][0][lane];
      const float l_b = xch_s[wv ^ 1][1][lane];
      const float m_a = fresh[0] ? kNegInf : m_ref[0];
      const float m = fmaxf(m_a, m_b);
      const float fa = m_a == kNegInf ? 0.0f : __builtin_amdgcn_exp2f(m_a - m);
      const float fb = m_b == kNegInf ? 0.0f : __builtin_amdgcn_exp2f(m_b - m);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        oacc[0][0][i] = oacc[0][0][i] * fa + part_a[i * 64 + lane] * fb;
        oacc[0][1][i] = oacc[0][1][i] * fa + part_b[i * 64 + lane] * fb;
      }
      l_run[0] = l_run[0] * fa + l_b * fb;
      set_ref(0, m == kNegInf ? 0.0f : m);
      __syncthreads();  // the partner has read this wavefront's rows: they may be refilled
    }
    const float l_tot = l_run[0] + __shfl_xor(l_run[0], 32);
    const bool ok = q_ok[0] && l_tot > 0.0f;
    const float inv = ok ? 1.0f / l_tot : 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { oacc[0][0][i] *= inv; oacc[0][1][i] *= inv; }
    return ok ? (m_ref[0] + __log2f(l_tot)) * kLn2 : 0.0f;
  };

  // ---- walk over the tile list ----
  f32x16 ost[2];  // normalised short-term output of group 0, parked while the long-term branch runs
  float lse_st = 0.0f;
  bool st_open = !dense;
  reset();
  auto close_st = [&](uint16_t *kx, uint16_t *vx) __attribute__((always_inline)) {
    lse_st = close_branch(kx, vx);
    ost[0] = oacc[0][0];
    ost[1] = oacc[0][1];
    reset();
    st_open = false;
  };
  // step t: prefetch tile t+1 into the other buffer pair, wait for this wavefront's own loads
  // of tile t (the 8 just issued stay in flight), process tile t.  With one V buffer: request
  // V of tile t, then K of tile t+1; K of tile t (requested a step ago) is there once at most
  // those 8 are outstanding, V of tile t is waited for inside the tile.
  int J_cur = first_J;
  int J_nxt = list_entry(tile_raw(min(1, n_all - 1)));
  auto step = [&](int t, uint16_t *k_cur, uint16_t *v_cur, uint16_t *k_nxt, uint16_t *v_nxt) __attribute__((always_inline)) {
    const int J_after = tile_raw(min(t + 2, n_all - 1));  // consumed at the end of this step
    const bool last = t + 1 >= n_all;
    if (V1) {
      stage(Vh, v_lane, 0u, Vs0, J_cur);
      if (!last) {
        stage(Kh, k_lane, 64u, k_nxt, J_nxt);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
      } else {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(4));
      }
    } else if (!last) {
      stage(Kh, k_lane, 64u, k_nxt, J_nxt);
      stage(Vh, v_lane, 0u, v_nxt, J_nxt);
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
    } else {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    tile(k_cur, V1 ? Vs0 : v_cur, J_cur, t < n_st, last);
    J_cur = J_nxt;
    J_nxt = list_entry(J_after);
    if (st_open && t + 1 >= n_st) close_st(k_cur, v_cur);  // the window tiles are done
  };
  for (int t = 0; t < n_all; t += 2) {
    step(t, Ks0, Vs0, Ks1, Vs1);
    if (t + 1 < n_all) step(t + 1, Ks1, Vs1, Ks0, Vs0);
  }
  const float lse_lt = close_branch(Ks0, Vs0);

  // ---- epilogue: gate (Eq. 18-19) and stores of this wavefront's own 32 rows ----
  // A lane holds 4 consecutive channels of ONE row per accumulator quad; stored directly, an
  // instruction would touch 32 rows with 16 or 32 bytes each.  The tiles go through this
  // wavefront's staging rows instead (free now, XOR-swizzled against bank conflicts) and leave
  // as whole rows: 256 contiguous bytes per 16 lanes (fp32), 128 per 8 lanes (bf16).
  const int row0 = qbase[0];  // first of the 32 rows
  int el = lane;  // opaque copy: keeps the store addressing out of the registers of the tile loop
  asm volatile("" : "+v"(el));
  const int elq = el & 31, elh = el >> 5;
  auto store_f32_rows = [&](float *dst, const f32x16 (&acc)[2], uint16_t *piece_a, uint16_t *piece_b)
                            __attribute__((always_inline)) {
    float *pa = reinterpret_cast<float *>(piece_a + wv * HALF);  // rows 0..15, 256 bytes each
    float *pb = reinterpret_cast<float *>(piece_b + wv * HALF);  // rows 16..31
    float *mine = elq < 16 ? pa : pb;
    const int rl = elq & 15;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int chunk = 8 * mb + 2 * g + elh;  // 16-byte chunk of the row
        *reinterpret_cast<float4 *>(mine + rl * 64 + ((chunk ^ rl) * 4)) =
            make_float4(acc[mb][4 * g], acc[mb][4 * g + 1], acc[mb][4 * g + 2], acc[mb][4 * g + 3]);
      }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = 4 * (i & 3) + (el >> 4), c = el & 15;
      const float4 v = *reinterpret_cast<const float4 *>((i < 4 ? pa : pb) + rr * 64 + ((c ^ rr) * 4));
      const int grow = row0 + 16 * (i >> 2) + rr;
      typedef float f32x4_t __attribute__((ext_vector_type(4)));
      const f32x4_t vv = {v.x, v.y, v.z, v.w};
      if (grow < p.L) __builtin_nontemporal_store(vv, reinterpret_cast<f32x4_t *>(dst + head + (size_t)grow * D + 4 * c));
    }
  };
  // o4(mb, g, e): the value of channel 32*mb + 8*g + 4*lh + e of this lane's row
  auto store_bf16_rows = [&](uint16_t *dst, auto o4, uint16_t *piece) __attribute__((always_inline)) {
    uint16_t *pt = piece + wv * HALF;  // 32 rows of 128 bytes
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = pack2_bf16(o4(mb, g, 0), o4(mb, g, 1));
        pk.y = pack2_bf16(o4(mb, g, 2), o4(mb, g, 3));
        const int chunk = 4 * mb + g;  // 16-byte chunk (8 channels); this lane fills half lh of it
        *reinterpret_cast<uint2 *>(pt + elq * D + ((chunk ^ (elq & 7)) * 8) + 4 * elh) = pk;
      }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = 8 * i + (el >> 3), c = el & 7;
      const uint4 v = *reinterpret_cast<const uint4 *>(pt + rr * D + ((c ^ (rr & 7)) * 8));
      const int grow = row0 + rr;
      if (grow < p.L) *reinterpret_cast<uint4 *>(dst + head + (size_t)grow * D + 8 * c) = v;
    }
  };
  const size_t lrow = (size_t)bh * p.L + iq[0];
  if (dense) {
    store_bf16_rows(O, [&](int mb, int g, int e) { return oacc[0][mb][4 * g + e]; }, Ks0);
    if (iq[0] < p.L && lh == 0 && lse_lt_out) lse_lt_out[lrow] = lse_lt;
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
      z = fmaf(a.x, oacc[0][mb][4 * g], z);
      z = fmaf(a.y, oacc[0][mb][4 * g + 1], z);
      z = fmaf(a.z, oacc[0][mb][4 * g + 2], z);
      z = fmaf(a.w, oacc[0][mb][4 * g + 3], z);
      z = fmaf(b.x, ost[mb][4 * g], z);
      z = fmaf(b.y, ost[mb][4 * g + 1], z);
      z = fmaf(b.z, ost[mb][4 * g + 2], z);
      z = fmaf(b.w, ost[mb][4 * g + 3], z);
    }
  z += __shfl_xor(z, 32);
  z += gate_b ? gate_b[h] : 0.0f;
  const float alpha = q_ok[0] ? 1.0f / (1.0f + __expf(-z)) : 0.0f;
  if (o_lt_out) {
    store_f32_rows(o_lt_out, oacc[0], Ks0, Ks1);
    store_f32_rows(o_st_out, ost, Vs0, V1 ? Ks0 : Vs1);
  }
  store_bf16_rows(O, [&](int mb, int g, int e) {
    return alpha * oacc[0][mb][4 * g + e] + (1.0f - alpha) * ost[mb][4 * g + e];
  }, Ks0);
  if (iq[0] < p.L && lh == 0) {
    if (lse_lt_out) lse_lt_out[lrow] = lse_lt;
    if (lse_st_out) lse_st_out[lrow] = lse_st;
  }
}

bool fwd_mfma_supported(const KParams &p, int dtype)
{
  return dtype == 1 && p.d == 64 && (p.b == 32 || p.b == 64) && !p.bidir &&
         (p.sblk == 0 || (is_pow2(p.sblk) && p.sblk <= p.b));
}

void launch_fwd_mfma(const KParams &p, const FwdArgs &a, hipStream_t st)
{
  if (p.b == 64) {  // block size 64: the four-wavefront kernel of mfma_fwd4.hip
    launch_fwd_mfma4(p, a, st);
    return;
  }
  const unsigned grid = (unsigned)(p.B * p.H * p.nq);
  auto u16 = [](const void *x) { return reinterpret_cast<const uint16_t *>(x); };
  auto go = [&](auto kernel, unsigned threads) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, st, u16(a.Q), u16(a.K), u16(a.V), a.valid_len, a.sel,
                       a.gate_w, a.gate_b, (uint16_t *)a.O, (float *)a.o_lt, (float *)a.o_st, a.lse_lt, a.lse_st,
                       a.dense, p);
  };
  const bool eq15 = p.sblk != 0 && !a.dense;
  const bool sub = eq15 && p.sblk < p.b;  // mask block smaller than the tile
  if (p.b == 32) {
    if (sub) go(fwd_mfma_kernel<32, true, true>, 64);
    else if (eq15) go(fwd_mfma_kernel<32, true, false>, 64);
    else go(fwd_mfma_kernel<32, false, false>, 64);
  } else {
    if (sub) go(fwd_mfma_kernel<64, true, true>, 128);
    else if (eq15) go(fwd_mfma_kernel<64, true, false>, 128);
    else go(fwd_mfma_kernel<64, false, false>, 128);
  }
}

}  // namespace blossom

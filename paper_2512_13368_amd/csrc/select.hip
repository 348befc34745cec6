// Long-term block selection (Sec. 3.4): block compression (Eq. 9, phi = mean over the
// block's valid keys), importance scores (Eq. 10) and top-k (Eq. 13).
//
// The scores decide integers, so their arithmetic is fixed exactly: sequential fp32 sums in
// ascending position, one IEEE division, one fused-multiply-add chain over the channels.
// This file is compiled with -ffp-contract=off; the only fused operations are the explicit
// __fmaf_rn calls.  Plain ALUs only: the work is O(NB^2 d) per head and HBM-bound on the
// pooling pass.
#include "common.h"
#include "launch.h"

namespace blossom {

// ---- pooling ------------------------------------------------------------------------------
// One lane owns 4 channels of one block of one tensor and walks the block's valid positions
// in ascending order.  qsum  [B,H,NB,d]   (unnormalised sums of Q)
//                     kmeanT[B,H,d,NB]   (means of K, transposed so that the scoring pass
//                                         reads consecutive blocks with consecutive lanes)
// KCMP: K holds compressed keys [B,H,NB,d] supplied by the caller (Eq. 9 with the caller's phi);
// they are copied as they are into the transposed fp32 layout instead of being pooled.
template <typename T, int D, bool KCMP>
__global__ __launch_bounds__(256) void pool_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                   const int *__restrict__ valid_len,
                                                   float *__restrict__ qsum, float *__restrict__ kmeanT,
                                                   KParams p)
{
  constexpr int LPT = D / 4;  // lanes per (tensor, row-head, block) task
  const long n_bhj = (long)p.B * p.H * p.NB;
  const long task = (long)blockIdx.x * (256 / LPT) + threadIdx.x / LPT;
  if (task >= 2 * n_bhj) return;
  const int c4 = (threadIdx.x % LPT) * 4;
  const int which = task >= n_bhj;
  const long rem = which ? task - n_bhj : task;
  const int bh = (int)(rem / p.NB);
  const int J = (int)(rem % p.NB);
  if (!which && J < p.NB - p.nq) return;  // serving mode: only the last query block is pooled
  if (KCMP && which) {
    float x[4];
    load4(K + ((size_t)bh * p.NB + J) * D + c4, x);
#pragma unroll
    for (int e = 0; e < 4; ++e) kmeanT[((size_t)bh * D + c4 + e) * p.NB + J] = x[e];
    return;
  }
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  const int lo = max(J * p.b, p0);
  const int hi = min((J + 1) * p.b, p.L);
  const T *src = (which ? K : Q) + (size_t)bh * p.L * D + c4;
  float a[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
  for (int t = lo; t < hi; ++t) {
    float x[4];
    load4(src + (size_t)t * D, x);
    a[0] = a[0] + x[0];
    a[1] = a[1] + x[1];
    a[2] = a[2] + x[2];
    a[3] = a[3] + x[3];
  }
  if (!which) {
    store4(qsum + ((size_t)bh * p.NB + J) * D + c4, a);
  } else {
    const int cnt = hi - lo;
    const float fc = (float)cnt;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float m = cnt > 0 ? __fdiv_rn(a[e], fc) : 0.0f;
      kmeanT[((size_t)bh * D + c4 + e) * p.NB + J] = m;
    }
  }
}

// ---- pooling with the rotary position embedding applied on the way in (Sec. 3.3) ------------
// Every position (padding too) is rotated with the caller's cos/sin tables, rounded to the storage
// type and written to Q_rot / K_rot; the pooled sums are taken over those rounded values, so that
// selection, forward and backward all see the same rotated tensors.  Fixed fp32 recipe on channel
// pairs (2i, 2i+1) at position m: t = x1*s; x0' = fma(x0, c, -t); u = x1*c; x1' = fma(x0, s, u).
//
// One workgroup per (tensor, row-head, run of kRopeRows positions): the run is one contiguous chunk
// of memory, read and written with 16 bytes per lane, consecutive lanes on consecutive addresses.
// The rotated values also go to LDS (fp32), from where one thread per (block of the run, channel)
// takes the block's sum in ascending position order.
constexpr int kRopeRows = 64;

template <typename T, int D>
__global__ __launch_bounds__(256) void rope_pool_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                        const int *__restrict__ valid_len,
                                                        float *__restrict__ qsum, float *__restrict__ kmeanT,
                                                        T *__restrict__ Q_rot, T *__restrict__ K_rot, KParams p)
{
  constexpr int EPT = 16 / (int)sizeof(T);  // elements of a 16-byte piece: 8 bf16 or 4 fp32
  constexpr int PPR = D / EPT;              // pieces per row
  __shared__ __attribute__((aligned(16))) float rot_s[kRopeRows][D];  // (rows are read with one channel per lane: no padding needed)
  const int runs = (p.L + kRopeRows - 1) / kRopeRows;
  const int BH = p.B * p.H;
  const int which = blockIdx.x >= (unsigned)(BH * runs);
  const int rem = (int)blockIdx.x - which * BH * runs;
  const int bh = rem / runs, run = rem % runs;
  const int t_lo = run * kRopeRows, t_hi = min(t_lo + kRopeRows, p.L);
  const int J_lo = t_lo / p.b, J_hi = (t_hi - 1) / p.b;  // blocks of the run (kRopeRows is a multiple of every b)
  if (!which && J_hi < p.NB - p.nq) return;              // serving mode: queries of the last block only
  const T *src = (which ? K : Q) + ((size_t)bh * p.L + t_lo) * D;
  T *dst = (which ? K_rot : Q_rot) + ((size_t)bh * p.L + t_lo) * D;
  const int pieces = (t_hi - t_lo) * PPR;
  for (int q = threadIdx.x; q < pieces; q += 256) {
    const int r = q / PPR, c0 = (q % PPR) * EPT;
    const int t = t_lo + r;
    float x[EPT], y[EPT], cs[EPT / 2], sn[EPT / 2];
    if constexpr (EPT == 8) {
      load4(src + (size_t)q * EPT, reinterpret_cast<float(&)[4]>(x[0]));
      load4(src + (size_t)q * EPT + 4, reinterpret_cast<float(&)[4]>(x[4]));
      const float4 c = *reinterpret_cast<const float4 *>(p.rope_cos + (size_t)t * (D / 2) + c0 / 2);
      const float4 s4 = *reinterpret_cast<const float4 *>(p.rope_sin + (size_t)t * (D / 2) + c0 / 2);
      cs[0] = c.x; cs[1] = c.y; cs[2] = c.z; cs[3] = c.w;
      sn[0] = s4.x; sn[1] = s4.y; sn[2] = s4.z; sn[3] = s4.w;
    } else {
      load4(src + (size_t)q * EPT, reinterpret_cast<float(&)[4]>(x[0]));
      const float2 c = *reinterpret_cast<const float2 *>(p.rope_cos + (size_t)t * (D / 2) + c0 / 2);
      const float2 s2 = *reinterpret_cast<const float2 *>(p.rope_sin + (size_t)t * (D / 2) + c0 / 2);
      cs[0] = c.x; cs[1] = c.y;
      sn[0] = s2.x; sn[1] = s2.y;
    }
#pragma unroll
    for (int i = 0; i < EPT / 2; ++i) {
      y[2 * i] = __fmaf_rn(x[2 * i], cs[i], -__fmul_rn(x[2 * i + 1], sn[i]));
      y[2 * i + 1] = __fmaf_rn(x[2 * i], sn[i], __fmul_rn(x[2 * i + 1], cs[i]));
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) y[e] = to_f32(from_f32<T>(y[e]));  // what the attention kernels will read
#pragma unroll
    for (int e = 0; e < EPT; e += 4)
      *reinterpret_cast<float4 *>(&rot_s[r][c0 + e]) = make_float4(y[e], y[e + 1], y[e + 2], y[e + 3]);
    store4(dst + (size_t)q * EPT, reinterpret_cast<float(&)[4]>(y[0]));
    if constexpr (EPT == 8) store4(dst + (size_t)q * EPT + 4, reinterpret_cast<float(&)[4]>(y[4]));
  }
  __syncthreads();
  const int p0 = p.L - clamp_len(valid_len[bh / p.H], p.L);
  const int nblk = J_hi - J_lo + 1;
  for (int e = threadIdx.x; e < nblk * D; e += 256) {
    const int J = J_lo + e / D, c = e % D;
    if (!which && J < p.NB - p.nq) continue;
    const int lo = max(J * p.b, p0), hi = min((J + 1) * p.b, p.L);
    float a = 0.0f;
#pragma unroll 8
    for (int t = lo; t < hi; ++t) a = a + rot_s[t - t_lo][c];
    if (!which) {
      qsum[((size_t)bh * p.NB + J) * D + c] = a;
    } else {
      const int cnt = hi - lo;
      kmeanT[((size_t)bh * D + c) * p.NB + J] = cnt > 0 ? __fdiv_rn(a, (float)cnt) : 0.0f;
    }
  }
}

// ---- scoring + top-k ----------------------------------------------------------------------
// One wavefront per (row, head, query block I).  Lane-strided candidates J_first <= J < I.
// Each score becomes one 64-bit key in LDS: an order-preserving integer image of the fp32 score
// (with -0 folded onto +0, so that equal scores give equal images) above NB-1-J, so that
// "beats" under (score descending, index ascending) is a single unsigned comparison of unique
// keys.  A candidate is selected iff fewer than `take` candidates beat it; ballots and prefix
// popcounts emit the list in ascending order.
__device__ __forceinline__ unsigned long long rank_key(float score, int J, int NB)
{
  unsigned u = __float_as_uint(score);
  if (u == 0x80000000u) u = 0u;                       // -0 ties with +0
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);     // monotone in the score
  return ((unsigned long long)u << 32) | (unsigned)(NB - 1 - J);
}

template <int D>
__global__ __launch_bounds__(64) void score_topk_kernel(const float *__restrict__ qsum,
                                                        const float *__restrict__ kmeanT,
                                                        const int *__restrict__ valid_len,
                                                        int *__restrict__ sel, KParams p)
{
  __shared__ float qs[D];
  extern __shared__ unsigned long long key_s[];  // NB keys (sized at launch: a static worst-case array would cap the occupancy)
  const int lane = threadIdx.x;
  const int I = p.NB - p.nq + (int)(blockIdx.x % p.nq);
  const int bh = blockIdx.x / p.nq;
  const int n = clamp_len(valid_len[bh / p.H], p.L);
  const int p0 = p.L - n;
  int *out = sel + ((size_t)bh * p.NB + I) * p.k;
  const int hi = min((I + 1) * p.b, p.L);
  if (hi <= p0) {  // no valid query in this block
    for (int e = lane; e < p.k; e += 64) out[e] = -1;
    return;
  }
  const int J_first = p0 / p.b;
  // candidates: the earlier blocks that hold a valid key; in the bidirectional form the later ones too.
  // There the query's own block sits among them with the largest possible key, so it is always taken
  // and comes out at its place in the ascending list.
  const int J_end = p.bidir ? p.NB : I;
  const int n_cand = p.bidir ? p.NB - J_first - 1 : I - J_first;
  const int take = min(p.k - 1, n_cand) + (p.bidir ? 1 : 0);
  for (int c = lane; c < D; c += 64) qs[c] = qsum[((size_t)bh * p.NB + I) * D + c];
  __syncthreads();
  const float *km = kmeanT + (size_t)bh * D * p.NB;
  if (J_end - J_first <= 128 && J_end - J_first > 40) {  // (fewer candidates: the rank loop below is cheaper)
    // Up to two candidates per lane, kept in registers.  Their scores are two independent chains over
    // the channels; the k-th largest score image is found by a radix search from the top bit down
    // (one ballot and one population count per bit and candidate slot: scalar work), and equal
    // images are taken in ascending block order, which is the lower-index-wins rule.
    const int Ja = J_first + lane, Jb = Ja + 64;
    const bool has_a = Ja < J_end, has_b = Jb < J_end;
    float acc_a = 0.0f, acc_b = 0.0f;
    const float *ka = km + min(Ja, p.NB - 1), *kb = km + min(Jb, p.NB - 1);
    if (J_end - J_first > 64) {
#pragma unroll 16
      for (int c = 0; c < D; ++c) {
        acc_a = __fmaf_rn(qs[c], ka[(size_t)c * p.NB], acc_a);
        acc_b = __fmaf_rn(qs[c], kb[(size_t)c * p.NB], acc_b);
      }
    } else {
#pragma unroll 16
      for (int c = 0; c < D; ++c) acc_a = __fmaf_rn(qs[c], ka[(size_t)c * p.NB], acc_a);
    }
    // 32-bit image of rank_key's upper word; the own block (bidirectional form) gets the largest value
    auto image = [&](float sc, int J) -> unsigned {
      if (J == I) return 0xFFFFFFFFu;
      return (unsigned)(rank_key(sc, 0, 1) >> 32);
    };
    const unsigned ua = image(acc_a, Ja), ub = image(acc_b, Jb);
    unsigned prefix = 0;
    int remaining = take;
    if (take > 0) {
      for (int bit = 31; bit >= 0; --bit) {
        const unsigned test = prefix | (1u << bit);
        const unsigned himask = ~((1u << bit) - 1u);
        const int cnt = __popcll(__ballot(has_a && (ua & himask) == test)) +
                        __popcll(__ballot(has_b && (ub & himask) == test));
        if (cnt >= remaining) prefix = test;  // the k-th largest has this bit set
        else remaining -= cnt;                // everything with this bit set lies above it
      }
    }
    // prefix: the take-th largest image; `remaining` of the candidates equal to it are still to be taken
    const unsigned long long eq_a = __ballot(has_a && ua == prefix), eq_b = __ballot(has_b && ub == prefix);
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    const bool ch_a = take > 0 && has_a && (ua > prefix || (ua == prefix && __popcll(eq_a & lt_mask) < remaining));
    const bool ch_b = take > 0 && has_b &&
                      (ub > prefix || (ub == prefix && __popcll(eq_a) + __popcll(eq_b & lt_mask) < remaining));
    const unsigned long long ma = __ballot(ch_a), mb = __ballot(ch_b);
    if (ch_a) out[__popcll(ma & lt_mask)] = Ja;
    const int na = __popcll(ma);
    if (ch_b) out[na + __popcll(mb & lt_mask)] = Jb;
    int base = na + __popcll(mb);
    if (!p.bidir) {
      if (lane == 0) out[base] = I;
      ++base;
    }
    for (int e = base + lane; e < p.k; e += 64) out[e] = -1;
    return;
  }
  for (int J = J_first + lane; J < J_end; J += 64) {
    float acc = 0.0f;
#pragma unroll 8
    for (int c = 0; c < D; ++c) acc = __fmaf_rn(qs[c], km[(size_t)c * p.NB + J], acc);
    key_s[J] = J == I ? ~0ull : rank_key(acc, J, p.NB);
  }
  __syncthreads();
  int base = 0;
  for (int J0 = J_first; J0 < J_end; J0 += 64) {
    const int J = J0 + lane;
    bool chosen = false;
    if (J < J_end) {
      const unsigned long long mine = key_s[J];
      int rank = 0;
      for (int Jo = J_first; Jo < J_end; ++Jo) rank += key_s[Jo] > mine ? 1 : 0;
      chosen = rank < take;
    }
    const unsigned long long mask = __ballot(chosen);
    if (chosen) {
      const unsigned long long below = mask & ((1ull << lane) - 1ull);
      out[base + __popcll(below)] = J;
    }
    base += __popcll(mask);
  }
  // base == take here; causal form: the own block closes the list; the rest is padding
  if (!p.bidir) {
    if (lane == 0) out[base] = I;
    ++base;
  }
  for (int e = base + lane; e < p.k; e += 64) out[e] = -1;
}

// ---- launchers ----------------------------------------------------------------------------
template <typename T, int D>
static void launch_select_t(const KParams &p, const void *Q, const void *K, bool kcmp, const int *valid_len,
                            int *sel, void *ws, void *Q_rot, void *K_rot, hipStream_t st)
{
  float *qsum = reinterpret_cast<float *>(ws);
  float *kmeanT = qsum + (size_t)p.B * p.H * p.NB * D;
  const long tasks = 2L * p.B * p.H * p.NB;
  const int per_wg = 256 / (D / 4);
  const unsigned grid = (unsigned)((tasks + per_wg - 1) / per_wg);
  if (kcmp) {
    BLOSSOM_LAUNCH((pool_kernel<T, D, true>), dim3(grid), dim3(256), 0, st, (const T *)Q, (const T *)K,
                   valid_len, qsum, kmeanT, p);
  } else if (p.rope_cos) {
    const long rgrid = 2L * p.B * p.H * ((p.L + kRopeRows - 1) / kRopeRows);
    BLOSSOM_LAUNCH((rope_pool_kernel<T, D>), dim3((unsigned)rgrid), dim3(256), 0, st,
                   (const T *)Q, (const T *)K, valid_len, qsum, kmeanT, (T *)Q_rot, (T *)K_rot, p);
  } else {
    BLOSSOM_LAUNCH((pool_kernel<T, D, false>), dim3(grid), dim3(256), 0, st, (const T *)Q, (const T *)K,
                   valid_len, qsum, kmeanT, p);
  }
  hipLaunchKernelGGL((score_topk_kernel<D>), dim3((unsigned)(p.B * p.H * p.nq)), dim3(64),
                     (size_t)p.NB * sizeof(unsigned long long), st,
                     qsum, kmeanT, valid_len, sel, p);
}

size_t select_workspace_bytes(const KParams &p) { return 2 * (size_t)p.B * p.H * p.NB * p.d * sizeof(float); }

void launch_select(const KParams &p, int dtype, const void *Q, const void *K, bool kcmp, const int *valid_len,
                   int *sel, void *ws, hipStream_t st, void *Q_rot, void *K_rot)
{
  with_head_dim(p.d, [&](auto dim) {
    constexpr int D = decltype(dim)::value;
    if (dtype == 0) launch_select_t<float, D>(p, Q, K, kcmp, valid_len, sel, ws, Q_rot, K_rot, st);
    else launch_select_t<bf16_t, D>(p, Q, K, kcmp, valid_len, sel, ws, Q_rot, K_rot, st);
  });
}

}  // namespace blossom

// The selection rule of Sec. 3.4 as the paper prints it (Eq. 8-13): overlapping compression blocks,
// per-position softmax scores over the compression blocks, the score mapping of Eq. 11, the sum over
// the query heads that share a key/value head (Eq. 12, grouped-query attention of Eq. 4-5), and the
// top-k selection blocks per query position and group (Eq. 13).
//
// The result is a set of integers, so the arithmetic is fixed exactly (this file is compiled with
// -ffp-contract=off; fused operations are only the explicit __fmaf_rn calls): sums ascending from
// +0.0f, dot products as fused-multiply-add chains over the channels, one multiply by the score
// scale, x - max, the exponential canon_exp below, the softmax normaliser as ONE sequential sum in
// ascending block order, one IEEE division per score, Eq. 11 in its printed loop order, heads in
// ascending order.  Plain ALUs only.
#include "../../include/blossom.h"

#include "common.h"
#include "launch.h"

namespace blossom {

namespace {

constexpr int kPosSlots = 8;  // candidate selection blocks per lane: up to 512 blocks before a position

// exp(x) for x <= 0, the same steps on every machine: y = x*log2(e) (one multiply), n = rint(y) (ties
// to even), f = y - n (exact), 2^f by the degree-7 Taylor polynomial of e^(f ln 2) in Horner form,
// scaled by 2^n exactly; 0 below the normal range.
__device__ __forceinline__ float canon_exp(float x)
{
  const float y = __fmul_rn(x, 1.44269502f);
  const float n = rintf(y);
  if (n < -125.0f) return 0.0f;
  const float f = __fsub_rn(y, n);
  float pz = 1.52527338e-05f;
  pz = __fmaf_rn(pz, f, 0.000154035304f);
  pz = __fmaf_rn(pz, f, 0.00133335581f);
  pz = __fmaf_rn(pz, f, 0.00961812911f);
  pz = __fmaf_rn(pz, f, 0.0555041087f);
  pz = __fmaf_rn(pz, f, 0.240226507f);
  pz = __fmaf_rn(pz, f, 0.693147182f);
  pz = __fmaf_rn(pz, f, 1.0f);
  return ldexpf(pz, (int)n);
}

// order-preserving 32-bit image of a score (-0 folded onto +0)
__device__ __forceinline__ unsigned score_image(float sc)
{
  unsigned u = __float_as_uint(sc);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct PosParams {
  int B, H, G, L, d;
  int l, s, lsel;   // compression block, stride, selection block
  int k;            // blocks per position, own block included
  int M, NBs;       // compression blocks, selection blocks
  float fscale;
};

// ---- Eq. 8-9: compressed keys, transposed: kcmpT [B*G][d][M] ----
template <typename T, int D>
__global__ __launch_bounds__(256) void cmp_pool_kernel(const T *__restrict__ K, const int *__restrict__ valid_len,
                                                       float *__restrict__ kcmpT, PosParams p)
{
  constexpr int LPT = D / 4;
  const long task = (long)blockIdx.x * (256 / LPT) + threadIdx.x / LPT;
  if (task >= (long)p.B * p.G * p.M) return;
  const int c4 = (threadIdx.x % LPT) * 4;
  const int bg = (int)(task / p.M), m = (int)(task % p.M);
  const int p0 = p.L - clamp_len(valid_len[bg / p.G], p.L);
  const int lo = max(m * p.s, p0), hi = m * p.s + p.l;  // (hi <= L by the definition of M)
  const T *src = K + (size_t)bg * p.L * D + c4;
  float a[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
  for (int t = lo; t < hi; ++t) {
    float x[4];
    load4(src + (size_t)t * D, x);
#pragma unroll
    for (int e = 0; e < 4; ++e) a[e] = a[e] + x[e];
  }
  const int cnt = hi - lo;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    kcmpT[((size_t)bg * D + c4 + e) * p.M + m] = cnt > 0 ? __fdiv_rn(a[e], (float)cnt) : 0.0f;
}

// ---- Eq. 10-13: one wavefront per (row, group, position) ----
template <typename T, int D>
__global__ __launch_bounds__(256) void pos_select_kernel(const T *__restrict__ Q, const float *__restrict__ kcmpT,
                                                         const int *__restrict__ valid_len, int *__restrict__ sel,
                                                         PosParams p)
{
  extern __shared__ float pos_lds[];  // per wavefront: D query values, then M scores
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const long item = (long)blockIdx.x * 4 + wv;
  if (item >= (long)p.B * p.G * p.L) return;
  const int bg = (int)(item / p.L), t = (int)(item % p.L);
  const int r = bg / p.G, g = bg % p.G;
  const int Hg = p.H / p.G;
  float *qs = pos_lds + (size_t)wv * (D + p.M + 1);
  float *es = qs + D;
  int *out = sel + ((size_t)bg * p.L + t) * p.k;
  const int p0 = p.L - clamp_len(valid_len[r], p.L);
  if (t < p0) {
    for (int e = lane; e < p.k; e += 64) out[e] = -1;
    return;
  }
  // eligible compression blocks: they end at or before t and hold a valid key
  int m_hi = -1;
  if (t - p.l + 1 >= 0) m_hi = min(p.M - 1, (t - p.l + 1) / p.s);
  const int need = p0 - p.l + 1;
  const int m_lo = need <= 0 ? 0 : (need + p.s - 1) / p.s;
  const int n_m = m_hi - m_lo + 1;
  const int jt = t / p.lsel, j_first = p0 / p.lsel;
  const int n_cand = jt - j_first;                 // candidates j_first .. jt-1
  const int ns = (n_cand + 63) / 64;               // slots in use (<= kPosSlots, checked at the boundary)
  const int ra = p.lsel / p.s, rc = p.l / p.s;
  float sgrp[kPosSlots];
#pragma unroll
  for (int u = 0; u < kPosSlots; ++u) sgrp[u] = 0.0f;
  const float *km = kcmpT + (size_t)bg * D * p.M;
  for (int hh = 0; hh < Hg; ++hh) {
    const T *qrow = Q + (((size_t)r * p.H + (size_t)g * Hg + hh) * p.L + t) * D;
    __builtin_amdgcn_wave_barrier();
    if (lane < D / 4) {
      float x[4];
      load4(qrow + 4 * lane, x);
#pragma unroll
      for (int e = 0; e < 4; ++e) qs[4 * lane + e] = x[e];
    }
    __builtin_amdgcn_wave_barrier();
    if (n_m > 0) {
      float mx = -__builtin_huge_valf();
      for (int m = m_lo + lane; m <= m_hi; m += 64) {  // Eq. 10: logits
        float acc = 0.0f;
#pragma unroll 8
        for (int c = 0; c < D; ++c) acc = __fmaf_rn(qs[c], km[(size_t)c * p.M + m], acc);
        const float x = __fmul_rn(acc, p.fscale);
        es[m - m_lo] = x;
        mx = fmaxf(mx, x);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      for (int m = m_lo + lane; m <= m_hi; m += 64) es[m - m_lo] = canon_exp(__fsub_rn(es[m - m_lo], mx));
      __builtin_amdgcn_wave_barrier();
      float z = 0.0f;  // the normaliser: one sequential sum, every lane takes it (same address: a broadcast read)
      for (int i = 0; i < n_m; ++i) z = z + es[i];
      __builtin_amdgcn_wave_barrier();
      for (int i = lane; i < n_m; i += 64) es[i] = __fdiv_rn(es[i], z);
      __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int u = 0; u < kPosSlots; ++u) {  // Eq. 11 for this lane's candidate blocks, Eq. 12 over the heads
      if (u < ns) {
        const int j = j_first + lane + 64 * u;
        float acc = 0.0f;
        if (j < jt)
          for (int a = 0; a < ra; ++a)
            for (int c = 0; c < rc; ++c) {
              const int idx = ra * j - a - c;
              if (idx >= m_lo && idx <= m_hi) acc = acc + es[idx - m_lo];
            }
        sgrp[u] = sgrp[u] + acc;
      }
    }
  }
  // Eq. 13: the own block and the best min(k-1, n_cand) earlier ones by (score descending, index ascending):
  // radix search for the k-th largest score image, equal images in ascending block order
  const int take = min(p.k - 1, n_cand);
  unsigned ui[kPosSlots];
  bool has[kPosSlots];
#pragma unroll
  for (int u = 0; u < kPosSlots; ++u) {
    has[u] = u < ns && j_first + lane + 64 * u < jt;
    ui[u] = score_image(sgrp[u]);
  }
  unsigned prefix = 0;
  int remaining = take;
  if (take > 0) {
    for (int bit = 31; bit >= 0; --bit) {
      const unsigned test = prefix | (1u << bit);
      const unsigned himask = ~((1u << bit) - 1u);
      int cnt = 0;
#pragma unroll
      for (int u = 0; u < kPosSlots; ++u)
        if (u < ns) cnt += __popcll(__ballot(has[u] && (ui[u] & himask) == test));
      if (cnt >= remaining) prefix = test;
      else remaining -= cnt;
    }
  }
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  int base = 0, eq_before = 0;
#pragma unroll
  for (int u = 0; u < kPosSlots; ++u) {
    if (u < ns) {
      const unsigned long long eq = __ballot(has[u] && ui[u] == prefix);
      const bool ch = take > 0 && has[u] &&
                      (ui[u] > prefix || (ui[u] == prefix && eq_before + __popcll(eq & lt_mask) < remaining));
      const unsigned long long cm = __ballot(ch);
      if (ch) out[base + __popcll(cm & lt_mask)] = j_first + lane + 64 * u;
      base += __popcll(cm);
      eq_before += __popcll(eq);
    }
  }
  if (lane == 0) out[base] = jt;
  for (int e = base + 1 + lane; e < p.k; e += 64) out[e] = -1;
}

// ---- Eq. 10-13 for short sequences: one LANE per position, a wavefront per 64 consecutive positions of a
// (row, group).  With at most 64 compression blocks and 64 selection blocks a position's whole chain fits one
// lane: logits, softmax, Eq. 11 and the group sums run as plain sequential loops in exactly the order of the
// arithmetic recipe above (so the integers are those of the wavefront-per-position kernel), the scores sit in an
// LDS column per lane (index*64 + lane: no bank conflicts), and the top-k is k-1 passes over the candidates.
// The compression-block index is the same in every lane of a step, so the compressed keys are broadcast loads.
constexpr int kLaneMaxBlocks = 64;

template <typename T, int D>
__global__ __launch_bounds__(64) void pos_select_lane_kernel(const T *__restrict__ Q, const float *__restrict__ kcmpT,
                                                             const int *__restrict__ valid_len, int *__restrict__ sel,
                                                             PosParams p)
{
  extern __shared__ float lane_lds[];  // [M][64] scores of the current head, then [NBs][64] group sums
  const int lane = threadIdx.x;
  const int chunks = (p.L + 63) / 64;
  const int bg = blockIdx.x / chunks;
  const int t = (blockIdx.x % chunks) * 64 + lane;
  const int r = bg / p.G, g = bg % p.G;
  const int Hg = p.H / p.G;
  float *es = lane_lds + lane;
  float *sg = lane_lds + (size_t)p.M * 64 + lane;
  const int p0 = p.L - clamp_len(valid_len[r], p.L);
  if (t >= p.L) return;
  int *out = sel + ((size_t)bg * p.L + t) * p.k;
  if (t < p0) {
    for (int e = 0; e < p.k; ++e) out[e] = -1;
    return;
  }
  int m_hi = -1;
  if (t - p.l + 1 >= 0) m_hi = min(p.M - 1, (t - p.l + 1) / p.s);
  const int need = p0 - p.l + 1;
  const int m_lo = need <= 0 ? 0 : (need + p.s - 1) / p.s;
  const int n_m = m_hi - m_lo + 1;
  const int jt = t / p.lsel, j_first = p0 / p.lsel;
  const int n_cand = jt - j_first;  // candidates j_first .. jt-1
  const int ra = p.lsel / p.s, rc = p.l / p.s;
  for (int j = 0; j < n_cand; ++j) sg[j * 64] = 0.0f;
  const float *km = kcmpT + (size_t)bg * D * p.M;
  for (int hh = 0; hh < Hg; ++hh) {
    const T *qrow = Q + (((size_t)r * p.H + (size_t)g * Hg + hh) * p.L + t) * D;
    float q[D];
#pragma unroll
    for (int c4 = 0; c4 < D / 4; ++c4) {
      float x[4];
      load4(qrow + 4 * c4, x);
#pragma unroll
      for (int e = 0; e < 4; ++e) q[4 * c4 + e] = x[e];
    }
    if (n_m > 0) {
      float mx = -__builtin_huge_valf();
      for (int m = m_lo; m <= m_hi; ++m) {  // Eq. 10: logits
        float acc = 0.0f;
#pragma unroll
        for (int c = 0; c < D; ++c) acc = __fmaf_rn(q[c], km[(size_t)c * p.M + m], acc);
        const float x = __fmul_rn(acc, p.fscale);
        es[(m - m_lo) * 64] = x;
        mx = fmaxf(mx, x);
      }
      float z = 0.0f;  // the normaliser: one sequential sum in ascending block order
      for (int i = 0; i < n_m; ++i) {
        const float e = canon_exp(__fsub_rn(es[i * 64], mx));
        es[i * 64] = e;
        z = z + e;
      }
      for (int i = 0; i < n_m; ++i) es[i * 64] = __fdiv_rn(es[i * 64], z);
    }
    for (int j = j_first; j < jt; ++j) {  // Eq. 11 in its printed loop order, Eq. 12 over the heads
      float acc = 0.0f;
      for (int a = 0; a < ra; ++a)
        for (int c = 0; c < rc; ++c) {
          const int idx = ra * j - a - c;
          if (idx >= m_lo && idx <= m_hi) acc = acc + es[(idx - m_lo) * 64];
        }
      sg[(j - j_first) * 64] = sg[(j - j_first) * 64] + acc;
    }
  }
  // Eq. 13: the own block and the best min(k-1, n_cand) earlier ones by (score descending, index ascending)
  const int take = min(p.k - 1, n_cand);
  unsigned long long chosen = 0ull;
  for (int pass = 0; pass < take; ++pass) {
    int best = -1;
    unsigned best_img = 0u;
    for (int j = 0; j < n_cand; ++j) {
      if ((chosen >> j) & 1ull) continue;
      const unsigned img = score_image(sg[j * 64]);
      if (best < 0 || img > best_img) {  // strictly greater: equal scores keep the lower index
        best = j;
        best_img = img;
      }
    }
    chosen |= 1ull << best;
  }
  int base = 0;
  for (int j = 0; j < n_cand; ++j)
    if ((chosen >> j) & 1ull) out[base++] = j_first + j;
  out[base++] = jt;
  for (; base < p.k; ++base) out[base] = -1;
}

int fill_pos_params(const blossom_params *p, int G, int l, int s, float score_scale, PosParams *pp)
{
  if (!p) return BLOSSOM_ERR_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1) return BLOSSOM_ERR_SHAPE;
  if (p->d != 8 && p->d != 16 && p->d != 32 && p->d != 64) return BLOSSOM_ERR_UNSUPPORTED;
  if (p->dtype != BLOSSOM_F32 && p->dtype != BLOSSOM_BF16) return BLOSSOM_ERR_UNSUPPORTED;
  if (G < 1 || p->H % G != 0) return BLOSSOM_ERR_PARAM;
  if (p->topk < 1 || p->block < 1 || l < 1 || s < 1 || l % s != 0 || p->block % s != 0) return BLOSSOM_ERR_PARAM;
  if (!(score_scale >= 0.0f) || !(score_scale < 3.0e38f)) return BLOSSOM_ERR_PARAM;
  const long NBs = ((long)p->L + p->block - 1) / p->block;
  if (NBs > 64L * kPosSlots) return BLOSSOM_ERR_SHAPE;  // candidates of a position must fit its lanes' slots
  if ((double)p->B * p->H * p->L * p->d > 9.0e18 || (long)p->B * G * p->L > 0x7FFFFFFFL * 4) return BLOSSOM_ERR_SHAPE;
  pp->B = p->B; pp->H = p->H; pp->G = G; pp->L = p->L; pp->d = p->d;
  pp->l = l; pp->s = s; pp->lsel = p->block; pp->k = p->topk;
  pp->M = p->L >= l ? (p->L - l) / s + 1 : 0;
  pp->NBs = (int)NBs;
  pp->fscale = score_scale > 0.0f ? score_scale : 1.0f;
  return BLOSSOM_OK;
}

template <typename T, int D>
void launch_pos(const PosParams &pp, const void *Q, const void *K, const int *valid_len, int *sel, float *kcmpT,
                hipStream_t st)
{
  if (pp.M > 0) {
    const long tasks = (long)pp.B * pp.G * pp.M;
    const int per_wg = 256 / (D / 4);
    BLOSSOM_LAUNCH((cmp_pool_kernel<T, D>), dim3((unsigned)((tasks + per_wg - 1) / per_wg)), dim3(256), 0, st,
                   (const T *)K, valid_len, kcmpT, pp);
  }
  if (pp.M <= kLaneMaxBlocks && pp.NBs <= kLaneMaxBlocks) {  // short sequences: a lane per position
    const unsigned chunks = (unsigned)((pp.L + 63) / 64);
    const size_t lds_lane = 64 * (size_t)(pp.M + pp.NBs) * sizeof(float);
    hipLaunchKernelGGL((pos_select_lane_kernel<T, D>), dim3((unsigned)(pp.B * pp.G) * chunks), dim3(64), lds_lane, st,
                       (const T *)Q, kcmpT, valid_len, sel, pp);
    return;
  }
  const long items = (long)pp.B * pp.G * pp.L;
  const size_t lds = 4 * (size_t)(D + pp.M + 1) * sizeof(float);
  hipLaunchKernelGGL((pos_select_kernel<T, D>), dim3((unsigned)((items + 3) / 4)), dim3(256), lds, st, (const T *)Q,
                     kcmpT, valid_len, sel, pp);
}

}  // namespace
}  // namespace blossom

using namespace blossom;

extern "C" {

size_t blossom_select_positions_workspace_bytes(const blossom_params *p, int32_t kv_groups, int32_t cmp_block,
                                                int32_t cmp_stride)
{
  PosParams pp;
  if (fill_pos_params(p, kv_groups, cmp_block, cmp_stride, 1.0f, &pp) != BLOSSOM_OK) return 0;
  return (size_t)pp.B * pp.G * pp.d * (size_t)(pp.M > 0 ? pp.M : 1) * sizeof(float);
}

int blossom_select_positions(const blossom_params *p, int32_t kv_groups, int32_t cmp_block, int32_t cmp_stride,
                             float score_scale, const void *Q, const void *K, const int32_t *valid_len,
                             int32_t *sel_pos, void *ws, size_t ws_bytes, void *hip_stream)
{
  PosParams pp;
  int rc = fill_pos_params(p, kv_groups, cmp_block, cmp_stride, score_scale, &pp);
  if (rc) return rc;
  if (!Q || !K || !valid_len || !sel_pos) return BLOSSOM_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(Q) & 15u) || (reinterpret_cast<uintptr_t>(K) & 15u)) return BLOSSOM_ERR_ALIGN;
  const size_t need = blossom_select_positions_workspace_bytes(p, kv_groups, cmp_block, cmp_stride);
  if (!ws || ws_bytes < need) return BLOSSOM_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return BLOSSOM_ERR_ALIGN;
  if (4 * (size_t)(pp.d + pp.M + 1) * sizeof(float) > 60 * 1024) return BLOSSOM_ERR_SHAPE;  // scores of a position in LDS
  (void)hipGetLastError();
  hipStream_t st = (hipStream_t)hip_stream;
  float *kcmpT = reinterpret_cast<float *>(ws);
  with_head_dim(pp.d, [&](auto dim) {
    constexpr int D = decltype(dim)::value;
    if (p->dtype == BLOSSOM_F32) launch_pos<float, D>(pp, Q, K, valid_len, sel_pos, kcmpT, st);
    else launch_pos<bf16_t, D>(pp, Q, K, valid_len, sel_pos, kcmpT, st);
  });
  return hipGetLastError() == hipSuccess ? BLOSSOM_OK : BLOSSOM_ERR_LAUNCH;
}

}  // extern "C"

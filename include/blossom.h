/*
 * blossom.h -- C ABI of libblossom.so: Blossom attention for MI355X (gfx950).
 *
 * Blossom attention (BlossomRec, arXiv 2512.13368, Sec. 3.3-3.6) replaces dense
 * causal self-attention in a Transformer sequential recommender by two sparse
 * branches and a gate:
 *   - long-term branch (LTIS, Sec. 3.4): key blocks are compressed (Eq. 9),
 *     scored against the query (Eq. 10), the top-k blocks are kept (Eq. 13) and
 *     attention runs over the keys of the kept blocks only (Eq. 14, 16);
 *   - short-term branch (STIS, Sec. 3.5): attention under a local mask
 *     (Eq. 15, 17): stis_mode 0 is the local-window term alone, stis_mode 1 the
 *     whole of Eq. 15 (window, whole blocks at power-of-two block distances, last
 *     block), both intersected with the causal mask j <= i; stis_mode 2 is Eq. 15
 *     as printed, symmetric, with no causal mask in either branch;
 *   - learnable gate (Sec. 3.6, Eq. 18-19): a sigmoid of a linear map of both
 *     branch outputs blends them.
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device unless a
 *     comment says "host".  `blossom_params` itself is read on the host.
 *   - Q, K, V, O, dO, dQ, dK, dV: [B,H,L,d], contiguous, d fastest, element type
 *     given by `dtype`, base address 16-byte aligned.  The saved branch outputs
 *     o_lt, o_st have the same shape but are ALWAYS fp32: backward forms
 *     D = dO_x.o_x from them, and rounding o_x to bf16 would leave an error of
 *     relative size 2^-9 |o_x| in every dS of the row, which dominates the
 *     gradient of rows that see only a few keys.
 *   - One block size `block` (b) serves as query-block, compression-block and
 *     selection-block size (Eq. 8 with l = s = l' = b, for which the score
 *     mapping of Eq. 11 is the identity).  NB = ceil(L/b); block I covers
 *     positions [I*b, min((I+1)*b, L)).
 *   - Row r of the batch has valid_len[r] valid positions, LEFT padded: valid
 *     positions are L-valid_len[r] .. L-1.  Values outside [0,L] are clamped.
 *     Pad queries give O = o_lt = o_st = 0 and lse = 0; pad keys are never read
 *     into a softmax or a pooled block; gradients of pad positions are 0.
 *   - Ownership: the caller owns every buffer, including the workspace.  The
 *     library allocates nothing, frees nothing and never synchronises; all work
 *     is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  Outputs are overwritten, never accumulated into.
 *   - Accuracy: against exact arithmetic on the same inputs, every output and gradient x obeys
 *     |x - ref| <= tol * (|ref| + rms(ref)) with tol = 1e-4 for BLOSSOM_F32 and 2e-2 for
 *     BLOSSOM_BF16 (bf16 storage and matrix-core operands, fp32 accumulation).  The bf16 bound
 *     is claimed for rows that attend up to 2048 keys per branch; the rounding noise of the
 *     bf16 probabilities grows with the square root of the keys per row, and beyond that range
 *     isolated near-zero gradient elements can leave the bound by a small factor.
 *   - Errors: 0 on success, a negative BLOSSOM_ERR_* otherwise.  All argument
 *     checks run before the first HIP call, so they work on a host with no GPU.
 *     No global state; thread-safe.  Inputs are assumed finite.
 */
#ifndef BLOSSOM_H_
#define BLOSSOM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  BLOSSOM_OK = 0,
  BLOSSOM_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  BLOSSOM_ERR_SHAPE = -2,       /* B, H or L < 1, or L/b too large (NB > 4096)                 */
  BLOSSOM_ERR_UNSUPPORTED = -3, /* d or b not in {8,16,32,64}, dtype, stis_mode; backward with
                                   last_block_only                                             */
  BLOSSOM_ERR_PARAM = -4,       /* topk < 1, window < 1, stis_block < 0, bad softmax_scale      */
  BLOSSOM_ERR_ALIGN = -5,       /* a tensor pointer is not 16-byte aligned                     */
  BLOSSOM_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than blossom_workspace_bytes()    */
  BLOSSOM_ERR_LAUNCH = -7,      /* a kernel launch failed (hipGetLastError)                    */
  BLOSSOM_ERR_TOO_LARGE = -8    /* blossom_select_blocks_static: scratch need beyond its maximum */
};

enum { BLOSSOM_F32 = 0, BLOSSOM_BF16 = 1 };
enum { BLOSSOM_WS_SELECT = 0, BLOSSOM_WS_FWD = 1, BLOSSOM_WS_BWD = 2, BLOSSOM_WS_DENSE = 3 };

typedef struct {
  int32_t B, H, L, d;     /* batch rows, heads, sequence length, head dimension                */
  int32_t block;          /* b                                                                  */
  int32_t topk;           /* k: blocks per query block INCLUDING its own (diagonal) block       */
  int32_t window;         /* w: query i sees keys j with 0 <= i-j < w in the short-term branch  */
  int32_t dtype;          /* BLOSSOM_F32 or BLOSSOM_BF16 (fp32 accumulation either way)         */
  float softmax_scale;    /* logits are softmax_scale * q.k ; 0.0f means 1/sqrt(d) (Eq. 1)      */
  int32_t stis_mode;      /* 0 = causal local window; 1 = causal form of Eq. 15 (see stis_block);
                             2 = bidirectional form, for backbones without a causal mask (Sec. 4.2):
                             Eq. 15 as printed, |i-j| < window or |b_q-b_k| = 2^r or j >= L - blk, with
                             mask block blk = stis_block (0 means `block`); the long-term branch takes its
                             k-1 candidates from the blocks on BOTH sides of the query block and sees the
                             selected blocks whole.  Every shape runs on the scalar kernels in this mode. */
  int32_t save_for_bwd;   /* fwd only: 1 = also write o_lt, o_st, lse_lt, lse_st                */
  int32_t stis_block;     /* stis_mode 1: mask block size blk of Eq. 15 (>= 1); 0 means `block`.
                             With b_q = i / blk, b_k = j / blk query i sees key j <= i iff
                             i - j < window, or b_q - b_k = 2^r for an integer r >= 0, or
                             j >= L - blk.  Ignored when stis_mode is 0.  (bf16, d = 64,
                             block 32 or 64 run on the matrix cores when blk is a power of two
                             not larger than block, e.g. the paper's blk = 1.)                   */
  int32_t last_block_only; /* 1: serving mode (Appendix C: only the representation of the last
                             position is scored).  blossom_select_blocks writes only the
                             selection row of the last query block, blossom_attn_fwd only the
                             rows of that block (O, and the saved tensors if asked for);
                             everything else in those buffers is left untouched.  Backward
                             calls return BLOSSOM_ERR_UNSUPPORTED.  0: all query blocks.          */
} blossom_params;

/* Bytes of device workspace an entry point needs (host call, no HIP).  `which` is a
 * BLOSSOM_WS_* value.  Returns 0 for invalid params or when no workspace is needed. */
size_t blossom_workspace_bytes(const blossom_params *p, int which);

/*
 * Long-term block selection (Sec. 3.4: Eq. 9 with phi = mean pooling, Eq. 10, Eq. 13).
 * For each (row, head, query block I) holding a valid query, writes the ascending list of
 * selected key blocks: block I itself plus the best min(k-1, I-J_first) earlier blocks
 * J_first <= J < I (J_first = first block holding a valid key), ordered by (score
 * descending, block index ascending); unused slots and blocks without a valid query hold -1.
 * The score of J for I is sum_c Qsum_I[c]*Kmean_J[c], evaluated in fp32 exactly as:
 * Qsum/Ksum = sequential sums over the block's valid positions in ascending order from
 * +0.0f; Kmean = Ksum/(float)count (IEEE division); score = fused multiply-add chain over
 * c = 0..d-1 from +0.0f.  +0.0 and -0.0 compare equal.
 *   Q, K        in   [B,H,L,d]
 *   valid_len   in   int32 [B]
 *   sel         out  int32 [B,H,NB,topk]
 *   ws          scratch, >= blossom_workspace_bytes(p, BLOSSOM_WS_SELECT), 16-byte aligned
 */
int blossom_select_blocks(const blossom_params *p, const void *Q, const void *K,
                          const int32_t *valid_len, int32_t *sel,
                          void *ws, size_t ws_bytes, void *hip_stream);

/*
 * blossom_select_blocks for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same arguments, checks, kernels and results as blossom_select_blocks, minus the
 * workspace: the pooled sums live in a static device array inside the library (16 MiB per GPU,
 * held until the process ends), whose device address is looked up once per GPU.  Calls no
 * hipMalloc/hipFree and no allocating routine.
 *   Limit: 8*B*H*ceil(L/block)*d bytes <= 16 MiB (16777216), else BLOSSOM_ERR_TOO_LARGE and
 *   nothing is launched (all five benchmark shapes fit: the largest needs 8 MiB).
 *   Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (different
 *   streams, different threads) race on it and must be ordered by the caller.  The array keeps
 *   the last call's contents; nothing in it needs clearing between calls, because the pooling
 *   pass writes every entry the scoring pass reads.
 */
int blossom_select_blocks_static(const blossom_params *p, const void *Q, const void *K,
                                 const int32_t *valid_len, int32_t *sel, void *hip_stream);

/*
 * The selection rule as the paper prints it (Sec. 3.4, Eq. 8-13), per query POSITION and key/value group
 * (grouped-query attention, Eq. 4-5: H query heads share G = kv_groups key heads, head h uses key head
 * h / (H/G)).  p->block is the selection block size l', p->topk is k, p->window and the stis fields are
 * not used.  Steps, all in a fixed fp32 arithmetic (sums ascending from +0, fused-multiply-add chains over
 * the channels, one sequential sum for the softmax normaliser, one IEEE division per score, a fixed
 * polynomial exponential), so that the integers that come out have one right answer:
 *   Eq. 8   compression block m covers positions [m*s, m*s+l), m < M = floor((L-l)/s)+1 (s | l, s | l';
 *           l may exceed l' as in the paper's own setting l = 32, s = 16, l' = 16);
 *   Eq. 9   compressed key = mean of the block's valid keys;
 *   Eq. 10  for position t: softmax over the compression blocks that end at or before t and hold a
 *           valid key of score_scale * q_t . Kcmp_m (score_scale 0 means 1, the printed formula);
 *   Eq. 11  S_sel[j] = sum_{a < l'/s} sum_{c < l/s} S_cmp[(l'/s) j - a - c];
 *   Eq. 12  the scores of the H/G query heads of a group are added;
 *   Eq. 13  the block holding t plus the best min(k-1, .) earlier selection blocks that hold a valid
 *           key, by (score descending, index ascending); ascending list, -1 padded; padding positions
 *           get all -1.
 *   Q        in   [B,H,L,d];  K in [B,G,L,d]  (element type p->dtype, 16-byte aligned)
 *   sel_pos  out  int32 [B,G,L,topk]
 *   ws       scratch, >= blossom_select_positions_workspace_bytes(...), 16-byte aligned
 * Limits: ceil(L/l') <= 512 selection blocks; BLOSSOM_ERR_SHAPE beyond.  (blossom_attn_fwd_positions below
 * consumes such a selection for short sequences; blossom_attn_fwd / blossom_attn_bwd take one selection row
 * per query block.)
 */
size_t blossom_select_positions_workspace_bytes(const blossom_params *p, int32_t kv_groups, int32_t cmp_block,
                                                int32_t cmp_stride);
int blossom_select_positions(const blossom_params *p, int32_t kv_groups, int32_t cmp_block, int32_t cmp_stride,
                             float score_scale, const void *Q, const void *K, const int32_t *valid_len,
                             int32_t *sel_pos, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Forward under a per-position selection (Sec. 3.4-3.6: Eq. 14 with the selection of Eq. 13 taken per query
 * position, Eq. 16-19; grouped-query attention, Eq. 4-5): the long-term branch of query position t of head h
 * attends the keys j <= t of the selection blocks listed in row [b, h / (H/G), t] of sel_pos; short-term
 * branch, gate and padding rules are those of blossom_attn_fwd (p->window, p->stis_mode 0 or 1, p->stis_block).
 * p->block is the selection block size l' (8 or 16), p->topk is k.
 *   Q               in   [B,H,L,d];  K, V in [B,G,L,d]  (element type p->dtype, 16-byte aligned), G = kv_groups | H
 *   sel_pos         in   int32 [B,G,L,topk]: ids of selection blocks or -1 (entries outside [0, ceil(L/l')) are
 *                        skipped), as blossom_select_positions writes them
 *   O               out  [B,H,L,d]
 *   o_lt, o_st      out  fp32 [B,H,L,d], or NULL;  lse_lt, lse_st  out  fp32 [B,H,L], or NULL
 * Served by the kernels that keep a head's K and V resident in LDS: d in {8, 16, 32}, l' in {8, 16}, at most 64
 * selection blocks, K and V of one (row, group) within 144 KB as fp32 rows (L <= 480 at d = 32, <= 900 at d <= 16);
 * BLOSSOM_ERR_UNSUPPORTED beyond, for stis_mode 2 and for last_block_only.  Needs no workspace.
 */
int blossom_attn_fwd_positions(const blossom_params *p, int32_t kv_groups, const void *Q, const void *K, const void *V,
                               const int32_t *valid_len, const int32_t *sel_pos, const float *gate_w,
                               const float *gate_b, void *O, void *o_lt, void *o_st, float *lse_lt, float *lse_st,
                               void *hip_stream);

/*
 * Backward of blossom_attn_fwd_positions (the gradients of Eq. 14, 16-19 under the per-position selection of
 * Eq. 13, grouped-query attention of Eq. 4-5), for training a model that takes the selection rule as printed.
 * Same formulas as blossom_attn_bwd with the long-term set of query position t read from row
 * [b, h / (H/G), t] of sel_pos; dK and dV of a key head are the sums over the H/G query heads that share it.
 *   Q, dO, dQ       [B,H,L,d];  K, V, dK, dV  [B,G,L,d]  (element type p->dtype, 16-byte aligned)
 *   sel_pos         in   int32 [B,G,L,topk], as given to the forward
 *   o_lt, o_st, lse_lt, lse_st   in   as the forward wrote them (all four required)
 *   d_gate_w        out  fp32 [H,2d];  d_gate_b  out fp32 [H] or NULL
 *   ws              scratch, >= blossom_workspace_bytes(p, BLOSSOM_WS_BWD), 16-byte aligned
 * Every output element is written (padding rows get zeros); no atomics, so results do not depend on timing.
 * Limits: those of blossom_attn_fwd_positions, with Q, dO and the per-position constants of one head within
 * 144 KB of LDS (L <= 432 at d = 32, <= 736 at d <= 16 with l' = 16; 64 blocks, L <= 512, with l' = 8); BLOSSOM_ERR_UNSUPPORTED beyond.
 */
int blossom_attn_bwd_positions(const blossom_params *p, int32_t kv_groups, const void *Q, const void *K, const void *V,
                               const int32_t *valid_len, const int32_t *sel_pos, const float *gate_w,
                               const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                               const float *lse_st, const void *dO, void *dQ, void *dK, void *dV, float *d_gate_w,
                               float *d_gate_b, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The layer around the attention, fused into one pass (Sec. 2.1 Eq. 4: the heads are concatenated and multiplied
 * by the output projection W^O; Sec. 3.6, the equation after Eq. 19: the result is added to the layer's input and
 * normalised, S = LayerNorm(H_prev + O_Blossom); dropout is the identity, as at inference):
 *   z[b,t,n] = H_prev[b,t,n] + bias[n] + sum_{h,e} O[b,h,t,e] * W_O_t[n, h*d + e]
 *   mean = sum_n z / d_model;  var = sum_n (z - mean)^2 / d_model;  rstd = 1 / sqrt(var + ln_eps)
 *   S[b,t,n] = (z - mean) * rstd * ln_gamma[n] + ln_beta[n]
 * O is read in the layout blossom_attn_fwd writes, so neither the concatenated heads, nor the projection's
 * output, nor the residual sum ever exist in memory.  Products and sums in fp32.  Every position is computed
 * (a padding row has O = 0 and gives LayerNorm(H_prev + bias)).  Of p only B, H, L, d and dtype are used (the
 * block must pass the same checks as for the other calls).
 *   O        in   [B,H,L,d]              element type p->dtype, 16-byte aligned
 *   W_O_t    in   [d_model, H*d]         p->dtype: row n holds column n of the printed W^O (the layout in which
 *                                         linear layers usually keep their weight, out-features x in-features)
 *   bias     in   fp32 [d_model] or NULL (the printed formula has none)
 *   H_prev   in   [B,L,d_model]          p->dtype
 *   ln_gamma, ln_beta   in  fp32 [d_model];  ln_eps >= 0
 *   S        out  [B,L,d_model]          p->dtype
 *   mean, rstd  out  fp32 [B,L] or NULL  (what a LayerNorm backward needs)
 * Shapes: bf16 with d = 64 and d_model 256 or 512 runs on the matrix cores; otherwise d_model a multiple of 8 up
 * to 1024 and H*d <= 1024 on scalar FMAs; BLOSSOM_ERR_UNSUPPORTED beyond.  Forward only: the backward of this
 * layer is two dense matrix products and stays with the caller.  Needs no workspace.
 */
int blossom_out_proj_ln(const blossom_params *p, int32_t d_model, const void *O, const void *W_O_t, const float *bias,
                        const void *H_prev, const float *ln_gamma, const float *ln_beta, float ln_eps, void *S,
                        float *mean, float *rstd, void *hip_stream);

/*
 * Rotary position embedding (Sec. 3.3: RoPE is applied to the projected Q and K before both branches)
 * fused into the pooling pass of blossom_select_blocks, which reads Q and K anyway: every position m of
 * every row is rotated on the way in, channel pairs (2i, 2i+1) by the angle of table entry [m][i],
 * rounded to the storage type and written to Q_rot / K_rot; the pooled sums, the scores and the
 * selection are those of the rotated tensors, which are what blossom_attn_fwd / blossom_attn_bwd_rope
 * then take as Q and K.  Against a separate rotation pass this saves one read of Q and of K.
 * Fixed fp32 recipe (the rotated bits decide the selection):
 *   t = x1*s;  x0' = fma(x0, c, -t);  u = x1*c;  x1' = fma(x0, s, u)     (c, s = cos, sin of the angle)
 *   rope_cos, rope_sin  in   fp32 [L, d/2], 16-byte aligned (e.g. the angles m * 10000^(-2i/d))
 *   Q_rot, K_rot        out  [B,H,L,d], element type as Q; padding positions are rotated too
 *   everything else as blossom_select_blocks.  With last_block_only, Q_rot holds the last query
 *   block only (K_rot is complete).
 */
int blossom_rope_select_blocks(const blossom_params *p, const void *Q, const void *K, const float *rope_cos,
                               const float *rope_sin, const int32_t *valid_len, void *Q_rot, void *K_rot,
                               int32_t *sel, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same selection with the block compression left to the caller (Sec. 3.4, Eq. 9: a learnable
 * phi): Kcmp holds one compressed key phi(K_J) per key block and takes the place of Kmean_J in
 * the score above, converted to fp32 as it is (rows of blocks before J_first are not read as
 * candidates).  Everything else (query sums, score recipe, ranking, output) is unchanged.
 *   Q           in   [B,H,L,d]
 *   Kcmp        in   [B,H,NB,d], element type and alignment as Q
 *   valid_len, sel, ws as above (same workspace size)
 */
int blossom_select_blocks_cmp(const blossom_params *p, const void *Q, const void *Kcmp,
                              const int32_t *valid_len, int32_t *sel,
                              void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Fused forward (Eq. 1 under the two masks, Eq. 16-19).  For every valid query i of block I:
 *   o_lt[i] = softmax over { j : block(j) in sel[I], j <= i, j valid } of scale*q_i.k_j, times V
 *   o_st[i] = softmax over { j : 0 <= i-j < window, j valid } of the same logits, times V
 *   alpha   = sigmoid( gate_w[h,0:d].o_lt[i] + gate_w[h,d:2d].o_st[i] + gate_b[h] )
 *   O[i]    = alpha*o_lt[i] + (1-alpha)*o_st[i]
 *   lse_x[i] = log sum exp of the branch's logits (natural log).
 *   sel        in   int32 [B,H,NB,topk] as written by blossom_select_blocks.  A row may also come
 *                   from the caller: its entries in [0,NB) must be distinct, and each query
 *                   block with a valid query must list itself; entries outside [0,NB) (such as
 *                   -1) are skipped wherever they stand in the row, and blocks after the query
 *                   block contribute nothing (causal mask).  Forward and backward read a row the
 *                   same way.
 *   gate_w     in   fp32 [H,2d];  gate_b in fp32 [H] or NULL (= 0)
 *   O          out  [B,H,L,d]
 *   o_lt,o_st  out  fp32 [B,H,L,d], lse_lt,lse_st out fp32 [B,H,L]; required iff save_for_bwd
 *   ws         scratch for BLOSSOM_WS_FWD (may be NULL when that size is 0)
 */
int blossom_attn_fwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                     const int32_t *valid_len, const int32_t *sel,
                     const float *gate_w, const float *gate_b,
                     void *O, void *o_lt, void *o_st, float *lse_lt, float *lse_st,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Backward of blossom_attn_fwd with the block selection held fixed (the top-k of Eq. 13 is
 * not differentiable).  Chain rule through Eq. 19, 18, 16/17 and Eq. 1:
 *   g = dO.(o_lt-o_st); dz = g*alpha*(1-alpha); d_gate_w[h] += dz*[o_lt;o_st]; d_gate_b[h] += dz
 *   dO_lt = alpha*dO + dz*gate_w[h,0:d];  dO_st = (1-alpha)*dO + dz*gate_w[h,d:2d]
 *   per branch x: D = dO_x.o_x; P = exp(S-lse_x); dV += P^T dO_x; dS = P*(dO_x V^T - D);
 *                 dQ += scale*dS K; dK += scale*dS^T Q
 *   o_lt,o_st,lse_lt,lse_st  in   as saved by the forward
 *   dO                       in   [B,H,L,d]
 *   dQ,dK,dV                 out  [B,H,L,d] (input dtype)
 *   d_gate_w                 out  fp32 [H,2d];  d_gate_b out fp32 [H] (may be NULL)
 * Results are deterministic: no floating-point atomics are used.
 */
int blossom_attn_bwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                     const int32_t *valid_len, const int32_t *sel,
                     const float *gate_w, const float *gate_b,
                     const void *o_lt, const void *o_st, const float *lse_lt, const float *lse_st,
                     const void *dO,
                     void *dQ, void *dK, void *dV, float *d_gate_w, float *d_gate_b,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * blossom_attn_bwd for Q and K that came out of blossom_rope_select_blocks (pass Q_rot, K_rot as Q, K):
 * dQ and dK are the gradients w.r.t. the tensors BEFORE the rotation, i.e. the kernels rotate every
 * gradient row back (the transpose rotation, in fp32, before rounding to the storage type) in their
 * store epilogues; no extra pass over dQ or dK.  dV and the gate gradients are unchanged.
 *   rope_cos, rope_sin  in   the tables given to blossom_rope_select_blocks
 */
int blossom_attn_bwd_rope(const blossom_params *p, const void *Q, const void *K, const void *V,
                          const int32_t *valid_len, const int32_t *sel,
                          const float *gate_w, const float *gate_b,
                          const void *o_lt, const void *o_st, const float *lse_lt, const float *lse_st,
                          const void *dO, const float *rope_cos, const float *rope_sin,
                          void *dQ, void *dK, void *dV, float *d_gate_w, float *d_gate_b,
                          void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The passes of blossom_attn_bwd one at a time, for profilers and benchmarks that need one
 * kernel per timed region.  Same arguments, workspace and checks as blossom_attn_bwd (of which
 * it is the general form: blossom_attn_bwd == all four bits); `stages` is a bit set:
 *   BLOSSOM_BWD_GATE     gate backward per row (Eq. 18-19) and reduction of d_gate_w, d_gate_b
 *   BLOSSOM_BWD_INVERSE  inverse selection list (key block -> query blocks that selected it)
 *   BLOSSOM_BWD_DQ       dQ
 *   BLOSSOM_BWD_DKV      dK and dV
 * A pass reads what earlier passes left in the workspace: DQ needs GATE; DKV needs GATE and
 * INVERSE, from calls with the same arguments and workspace.  Other bits are ignored.
 */
enum { BLOSSOM_BWD_GATE = 1, BLOSSOM_BWD_INVERSE = 2, BLOSSOM_BWD_DQ = 4, BLOSSOM_BWD_DKV = 8 };
int blossom_attn_bwd_stages(const blossom_params *p, const void *Q, const void *K, const void *V,
                            const int32_t *valid_len, const int32_t *sel,
                            const float *gate_w, const float *gate_b,
                            const void *o_lt, const void *o_st, const float *lse_lt, const float *lse_st,
                            const void *dO,
                            void *dQ, void *dK, void *dV, float *d_gate_w, float *d_gate_b,
                            void *ws, size_t ws_bytes, void *hip_stream, unsigned stages);

/*
 * Comparison kernel: dense causal attention over the valid suffix (Eq. 1 with the causal
 * mask), built in the same tile style.  topk, window, stis_mode and save_for_bwd are ignored.
 *   O out [B,H,L,d];  lse out fp32 [B,H,L] or NULL
 */
int blossom_dense_causal_fwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                             const int32_t *valid_len, void *O, float *lse,
                             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Measured ceilings of the matrix-core forward (Eq. 1 as tiled QK^T / softmax / PV for the
 * long-term and short-term branches, Eq. 16-17) on the GPU at hand: a stripped copy of its
 * steady-state tile loop for block size 64 and d = 64, with the same instruction mix and memory
 * access patterns but no masks, reference moves, tile list, prologue or epilogue.  A benchmark
 * times one launch and divides; no result is meaningful beyond "it ran".  The launch puts
 * BLOSSOM_PROBE_WORKGROUPS workgroups of two wavefronts on the chip (256 CUs x 4 resident x 4
 * rounds); every wavefront runs `iters` (even, >= 2) steps of 32 keys x 64 queries each.
 *   kind   0 matrix instructions only; 1 softmax VALU work only; 2 both, operands in registers;
 *          3 both, operands read from LDS; 4 the whole loop with global->LDS staging; 5 staging only
 *   K, V   in   bf16, blossom_probe_bytes(0) bytes each (contents: any finite values)
 *   sink   out  fp32, blossom_probe_bytes(1) bytes
 * Errors: BLOSSOM_ERR_NULL, BLOSSOM_ERR_PARAM (kind, iters), BLOSSOM_ERR_ALIGN, BLOSSOM_ERR_LAUNCH.
 */
#define BLOSSOM_PROBE_WORKGROUPS 4096
size_t blossom_probe_bytes(int which);
int blossom_probe(int kind, const void *K, const void *V, float *sink, int iters, void *hip_stream);

/* Static, human-readable text for an error code (host). */
const char *blossom_strerror(int code);

/* Library version string, e.g. "blossom-gfx950 0.1" (host). */
const char *blossom_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BLOSSOM_H_ */

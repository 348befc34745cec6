// C ABI of libblossom.so: argument validation (before any HIP call), workspace sizing and
// dispatch to the kernel launchers.  See include/blossom.h for the contract.
#include "../../include/blossom.h"

#include <cmath>
#include <mutex>

#include "launch.h"

using namespace blossom;

// Scratch of blossom_select_blocks_static: the pooled query sums and key means of one call.  Every
// GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

void *static_scratch_ptr()
{
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates the parameter block and fills the kernel-side description.
int check_params(const blossom_params *p, KParams *kp)
{
  if (!p) return BLOSSOM_ERR_NULL;
  if (p->B < 1 || p->H < 1 || p->L < 1) return BLOSSOM_ERR_SHAPE;
  if (p->d != 8 && p->d != 16 && p->d != 32 && p->d != 64) return BLOSSOM_ERR_UNSUPPORTED;
  if (p->block != 8 && p->block != 16 && p->block != 32 && p->block != 64) return BLOSSOM_ERR_UNSUPPORTED;
  if (p->dtype != BLOSSOM_F32 && p->dtype != BLOSSOM_BF16) return BLOSSOM_ERR_UNSUPPORTED;
  if (p->stis_mode < 0 || p->stis_mode > 2) return BLOSSOM_ERR_UNSUPPORTED;
  if (p->topk < 1 || p->window < 1) return BLOSSOM_ERR_PARAM;
  if (p->stis_mode >= 1 && p->stis_block < 0) return BLOSSOM_ERR_PARAM;
  if (!std::isfinite(p->softmax_scale) || p->softmax_scale < 0.0f) return BLOSSOM_ERR_PARAM;
  const long NB = ((long)p->L + p->block - 1) / p->block;
  if (NB > 4096) return BLOSSOM_ERR_SHAPE;
  if ((long)p->B * p->H * NB > 0x7FFFFFFFL) return BLOSSOM_ERR_SHAPE;
  if ((double)p->B * p->H * p->L * p->d > 9.0e18) return BLOSSOM_ERR_SHAPE;
  kp->B = p->B; kp->H = p->H; kp->L = p->L; kp->d = p->d;
  kp->b = p->block; kp->k = p->topk; kp->NB = (int)NB;
  kp->w = p->window < p->L ? p->window : p->L;  // a window beyond L sees the same keys as L: keeps i + w inside int
  kp->scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / std::sqrt((float)p->d);
  kp->sblk = p->stis_mode >= 1 ? (p->stis_block > 0 ? p->stis_block : p->block) : 0;
  kp->bidir = p->stis_mode == 2;
  kp->last_lo = kp->sblk > 0 ? p->L - kp->sblk : 0x3FFFFFFF;
  kp->nq = p->last_block_only ? 1 : (int)NB;
  kp->rope_cos = nullptr;
  kp->rope_sin = nullptr;
  return BLOSSOM_OK;
}

size_t ws_bytes_for(const KParams &kp, int dtype, int which)
{
  switch (which) {
    case BLOSSOM_WS_SELECT: return select_workspace_bytes(kp);
    case BLOSSOM_WS_FWD: return 0;
    case BLOSSOM_WS_BWD: return bwd_workspace_bytes(kp, dtype);
    case BLOSSOM_WS_DENSE: return 0;
    default: return 0;
  }
}

int check_ws(const KParams &kp, int dtype, int which, const void *ws, size_t ws_bytes)
{
  const size_t need = ws_bytes_for(kp, dtype, which);
  if (need == 0) return BLOSSOM_OK;
  if (!ws || ws_bytes < need) return BLOSSOM_ERR_WORKSPACE;
  if (!aligned16(ws)) return BLOSSOM_ERR_ALIGN;
  return BLOSSOM_OK;
}

// Called after the argument checks and before the first launch: drops an error that an unrelated
// earlier HIP call of the process left behind, so that launch_status() reports this call's own.
void clear_stale_error() { (void)hipGetLastError(); }

int launch_status()
{
  return hipGetLastError() == hipSuccess ? BLOSSOM_OK : BLOSSOM_ERR_LAUNCH;
}

}  // namespace

extern "C" {

size_t blossom_workspace_bytes(const blossom_params *p, int which)
{
  KParams kp;
  if (check_params(p, &kp) != BLOSSOM_OK) return 0;
  return ws_bytes_for(kp, p->dtype, which);
}

int blossom_select_blocks(const blossom_params *p, const void *Q, const void *K,
                          const int32_t *valid_len, int32_t *sel, void *ws, size_t ws_bytes,
                          void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (!Q || !K || !valid_len || !sel) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K)) return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_SELECT, ws, ws_bytes);
  if (rc) return rc;
  clear_stale_error();
  launch_select(kp, p->dtype, Q, K, false, valid_len, sel, ws, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_select_blocks_static(const blossom_params *p, const void *Q, const void *K,
                                 const int32_t *valid_len, int32_t *sel, void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (!Q || !K || !valid_len || !sel) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K)) return BLOSSOM_ERR_ALIGN;
  if (select_workspace_bytes(kp) > kStaticScratchBytes) return BLOSSOM_ERR_TOO_LARGE;
  void *ws = static_scratch_ptr();  // (first HIP call: after every argument check)
  if (!ws) return BLOSSOM_ERR_LAUNCH;
  clear_stale_error();
  // The pooling pass writes every entry the scoring pass reads, so nothing of the previous call's
  // contents has to be cleared.
  launch_select(kp, p->dtype, Q, K, false, valid_len, sel, ws, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_rope_select_blocks(const blossom_params *p, const void *Q, const void *K, const float *rope_cos,
                               const float *rope_sin, const int32_t *valid_len, void *Q_rot, void *K_rot,
                               int32_t *sel, void *ws, size_t ws_bytes, void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (!Q || !K || !rope_cos || !rope_sin || !valid_len || !Q_rot || !K_rot || !sel) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(Q_rot) || !aligned16(K_rot) || !aligned16(rope_cos) ||
      !aligned16(rope_sin))
    return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_SELECT, ws, ws_bytes);
  if (rc) return rc;
  kp.rope_cos = rope_cos;
  kp.rope_sin = rope_sin;
  clear_stale_error();
  launch_select(kp, p->dtype, Q, K, false, valid_len, sel, ws, (hipStream_t)hip_stream, Q_rot, K_rot);
  return launch_status();
}

int blossom_select_blocks_cmp(const blossom_params *p, const void *Q, const void *Kcmp,
                              const int32_t *valid_len, int32_t *sel, void *ws, size_t ws_bytes,
                              void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (!Q || !Kcmp || !valid_len || !sel) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(Kcmp)) return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_SELECT, ws, ws_bytes);
  if (rc) return rc;
  clear_stale_error();
  launch_select(kp, p->dtype, Q, Kcmp, true, valid_len, sel, ws, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_attn_fwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                     const int32_t *valid_len, const int32_t *sel, const float *gate_w,
                     const float *gate_b, void *O, void *o_lt, void *o_st, float *lse_lt,
                     float *lse_st, void *ws, size_t ws_bytes, void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (!Q || !K || !V || !valid_len || !sel || !gate_w || !O) return BLOSSOM_ERR_NULL;
  if (p->save_for_bwd && (!o_lt || !o_st || !lse_lt || !lse_st)) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return BLOSSOM_ERR_ALIGN;
  if (p->save_for_bwd && (!aligned16(o_lt) || !aligned16(o_st))) return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_FWD, ws, ws_bytes);
  if (rc) return rc;
  FwdArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.valid_len = valid_len; a.sel = sel;
  a.gate_w = gate_w; a.gate_b = gate_b; a.O = O;
  if (p->save_for_bwd) {
    a.o_lt = o_lt; a.o_st = o_st; a.lse_lt = lse_lt; a.lse_st = lse_st;
  }
  a.dense = 0;
  clear_stale_error();
  if (fwd_mfma_supported(kp, p->dtype)) launch_fwd_mfma(kp, a, (hipStream_t)hip_stream);
  else if (fwd_res_supported(kp, p->dtype)) launch_fwd_res(kp, p->dtype, a, (hipStream_t)hip_stream);
  else launch_fwd_generic(kp, p->dtype, a, (hipStream_t)hip_stream);
  return launch_status();
}

static int attn_bwd_impl(const blossom_params *p, const void *Q, const void *K, const void *V,
                         const int32_t *valid_len, const int32_t *sel, const float *gate_w,
                         const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                         const float *lse_st, const void *dO, void *dQ, void *dK, void *dV,
                         float *d_gate_w, float *d_gate_b, void *ws, size_t ws_bytes, void *hip_stream,
                         unsigned stages, const float *rope_cos, const float *rope_sin)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) return BLOSSOM_ERR_NULL;
  if (!aligned16(rope_cos) || !aligned16(rope_sin)) return BLOSSOM_ERR_ALIGN;
  kp.rope_cos = rope_cos;
  kp.rope_sin = rope_sin;
  if (p->last_block_only) return BLOSSOM_ERR_UNSUPPORTED;  // serving mode has no backward
  if (!Q || !K || !V || !valid_len || !sel || !gate_w || !o_lt || !o_st || !lse_lt || !lse_st ||
      !dO || !dQ || !dK || !dV || !d_gate_w)
    return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(o_lt) || !aligned16(o_st) ||
      !aligned16(dO) || !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
    return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_BWD, ws, ws_bytes);
  if (rc) return rc;
  BwdArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.valid_len = valid_len; a.sel = sel;
  a.gate_w = gate_w; a.gate_b = gate_b; a.o_lt = o_lt; a.o_st = o_st;
  a.lse_lt = lse_lt; a.lse_st = lse_st; a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV;
  a.d_gate_w = d_gate_w; a.d_gate_b = d_gate_b; a.ws = ws;
  clear_stale_error();
  launch_bwd(kp, p->dtype, a, stages & kBwdStageAll, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_attn_bwd_stages(const blossom_params *p, const void *Q, const void *K, const void *V,
                            const int32_t *valid_len, const int32_t *sel, const float *gate_w,
                            const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                            const float *lse_st, const void *dO, void *dQ, void *dK, void *dV,
                            float *d_gate_w, float *d_gate_b, void *ws, size_t ws_bytes, void *hip_stream,
                            unsigned stages)
{
  return attn_bwd_impl(p, Q, K, V, valid_len, sel, gate_w, gate_b, o_lt, o_st, lse_lt, lse_st, dO, dQ, dK, dV,
                       d_gate_w, d_gate_b, ws, ws_bytes, hip_stream, stages, nullptr, nullptr);
}

int blossom_attn_bwd_rope(const blossom_params *p, const void *Q, const void *K, const void *V,
                          const int32_t *valid_len, const int32_t *sel, const float *gate_w,
                          const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                          const float *lse_st, const void *dO, const float *rope_cos, const float *rope_sin,
                          void *dQ, void *dK, void *dV, float *d_gate_w, float *d_gate_b, void *ws,
                          size_t ws_bytes, void *hip_stream)
{
  if (!rope_cos || !rope_sin) return BLOSSOM_ERR_NULL;
  return attn_bwd_impl(p, Q, K, V, valid_len, sel, gate_w, gate_b, o_lt, o_st, lse_lt, lse_st, dO, dQ, dK, dV,
                       d_gate_w, d_gate_b, ws, ws_bytes, hip_stream, kBwdStageAll, rope_cos, rope_sin);
}

int blossom_attn_bwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                     const int32_t *valid_len, const int32_t *sel, const float *gate_w,
                     const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                     const float *lse_st, const void *dO, void *dQ, void *dK, void *dV,
                     float *d_gate_w, float *d_gate_b, void *ws, size_t ws_bytes, void *hip_stream)
{
  return blossom_attn_bwd_stages(p, Q, K, V, valid_len, sel, gate_w, gate_b, o_lt, o_st, lse_lt, lse_st, dO, dQ,
                                 dK, dV, d_gate_w, d_gate_b, ws, ws_bytes, hip_stream, kBwdStageAll);
}

int blossom_attn_fwd_positions(const blossom_params *p, int32_t kv_groups, const void *Q, const void *K, const void *V,
                               const int32_t *valid_len, const int32_t *sel_pos, const float *gate_w,
                               const float *gate_b, void *O, void *o_lt, void *o_st, float *lse_lt, float *lse_st,
                               void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (kv_groups < 1 || p->H % kv_groups != 0) return BLOSSOM_ERR_PARAM;
  if (!Q || !K || !V || !valid_len || !sel_pos || !gate_w || !O) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return BLOSSOM_ERR_ALIGN;
  if ((o_lt && !aligned16(o_lt)) || (o_st && !aligned16(o_st))) return BLOSSOM_ERR_ALIGN;
  if (!fwd_positions_supported(kp, p->dtype)) return BLOSSOM_ERR_UNSUPPORTED;
  FwdArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.valid_len = valid_len; a.sel = sel_pos;
  a.gate_w = gate_w; a.gate_b = gate_b; a.O = O;
  a.o_lt = o_lt; a.o_st = o_st; a.lse_lt = lse_lt; a.lse_st = lse_st;
  a.dense = 0;
  a.kv_groups = kv_groups;
  clear_stale_error();
  launch_fwd_res(kp, p->dtype, a, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_attn_bwd_positions(const blossom_params *p, int32_t kv_groups, const void *Q, const void *K, const void *V,
                               const int32_t *valid_len, const int32_t *sel_pos, const float *gate_w,
                               const float *gate_b, const void *o_lt, const void *o_st, const float *lse_lt,
                               const float *lse_st, const void *dO, void *dQ, void *dK, void *dV, float *d_gate_w,
                               float *d_gate_b, void *ws, size_t ws_bytes, void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (kv_groups < 1 || p->H % kv_groups != 0) return BLOSSOM_ERR_PARAM;
  if (!Q || !K || !V || !valid_len || !sel_pos || !gate_w || !o_lt || !o_st || !lse_lt || !lse_st || !dO || !dQ ||
      !dK || !dV || !d_gate_w)
    return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(o_lt) || !aligned16(o_st) || !aligned16(dO) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
    return BLOSSOM_ERR_ALIGN;
  if (!bwd_positions_supported(kp, p->dtype)) return BLOSSOM_ERR_UNSUPPORTED;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_BWD, ws, ws_bytes);
  if (rc) return rc;
  BwdArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.valid_len = valid_len; a.sel = sel_pos;
  a.gate_w = gate_w; a.gate_b = gate_b; a.o_lt = o_lt; a.o_st = o_st;
  a.lse_lt = lse_lt; a.lse_st = lse_st; a.dO = dO; a.dQ = dQ; a.dK = dK; a.dV = dV;
  a.d_gate_w = d_gate_w; a.d_gate_b = d_gate_b; a.ws = ws;
  clear_stale_error();
  // the per-row pass (gate gradient, the constants of each row) reads neither the selection nor K and V
  launch_bwd(kp, p->dtype, a, kBwdStageGate, (hipStream_t)hip_stream);
  if (launch_failed()) return launch_status();
  launch_bwd_positions(kp, p->dtype, a, bwd_carve(kp, p->dtype, ws), kv_groups, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_out_proj_ln(const blossom_params *p, int32_t d_model, const void *O, const void *W_O_t, const float *bias,
                        const void *H_prev, const float *ln_gamma, const float *ln_beta, float ln_eps, void *S,
                        float *mean, float *rstd, void *hip_stream)
{
  KParams kp;
  int rc = check_params(p, &kp);
  if (rc) return rc;
  if (d_model < 1 || !std::isfinite(ln_eps) || ln_eps < 0.0f) return BLOSSOM_ERR_PARAM;
  if (!O || !W_O_t || !H_prev || !ln_gamma || !ln_beta || !S) return BLOSSOM_ERR_NULL;
  if (!aligned16(O) || !aligned16(W_O_t) || !aligned16(H_prev) || !aligned16(S) || !aligned16(ln_gamma) ||
      !aligned16(ln_beta) || !aligned16(bias))
    return BLOSSOM_ERR_ALIGN;
  OutProjArgs a{};
  a.B = p->B; a.H = p->H; a.L = p->L; a.d = p->d; a.Dm = d_model; a.dtype = p->dtype;
  a.O = O; a.Wt = W_O_t; a.bias = bias; a.Hprev = H_prev; a.gamma = ln_gamma; a.beta = ln_beta; a.eps = ln_eps;
  a.S = S; a.mean = mean; a.rstd = rstd;
  if (!out_proj_supported(a)) return BLOSSOM_ERR_UNSUPPORTED;
  if ((double)p->B * p->L * d_model > 9.0e18) return BLOSSOM_ERR_SHAPE;
  clear_stale_error();
  launch_out_proj(a, (hipStream_t)hip_stream);
  return launch_status();
}

int blossom_dense_causal_fwd(const blossom_params *p, const void *Q, const void *K, const void *V,
                             const int32_t *valid_len, void *O, float *lse, void *ws,
                             size_t ws_bytes, void *hip_stream)
{
  blossom_params q;
  if (!p) return BLOSSOM_ERR_NULL;
  q = *p;
  q.topk = 1; q.window = 1; q.stis_mode = 0; q.stis_block = 0; q.save_for_bwd = 0;  // ignored fields
  q.last_block_only = 0;
  KParams kp;
  int rc = check_params(&q, &kp);
  if (rc) return rc;
  if (!Q || !K || !V || !valid_len || !O) return BLOSSOM_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return BLOSSOM_ERR_ALIGN;
  rc = check_ws(kp, p->dtype, BLOSSOM_WS_DENSE, ws, ws_bytes);
  if (rc) return rc;
  FwdArgs a{};
  a.Q = Q; a.K = K; a.V = V; a.valid_len = valid_len; a.O = O; a.lse_lt = lse;
  a.dense = 1;
  clear_stale_error();
  if (fwd_mfma_supported(kp, p->dtype)) launch_fwd_mfma(kp, a, (hipStream_t)hip_stream);
  else if (fwd_res_supported(kp, p->dtype)) launch_fwd_res(kp, p->dtype, a, (hipStream_t)hip_stream);
  else launch_fwd_generic(kp, p->dtype, a, (hipStream_t)hip_stream);
  return launch_status();
}

const char *blossom_strerror(int code)
{
  switch (code) {
    case BLOSSOM_OK: return "ok";
    case BLOSSOM_ERR_NULL: return "a required pointer is NULL";
    case BLOSSOM_ERR_SHAPE: return "bad shape: B, H, L must be >= 1 and ceil(L/block) <= 4096";
    case BLOSSOM_ERR_UNSUPPORTED: return "unsupported d, block, dtype or stis_mode, or backward in serving mode";
    case BLOSSOM_ERR_PARAM: return "bad parameter: topk >= 1, window >= 1, stis_block >= 0, finite softmax_scale >= 0";
    case BLOSSOM_ERR_ALIGN: return "tensor or workspace pointer not 16-byte aligned";
    case BLOSSOM_ERR_WORKSPACE: return "workspace missing or too small";
    case BLOSSOM_ERR_LAUNCH: return "kernel launch failed";
    case BLOSSOM_ERR_TOO_LARGE: return "problem too large for the static scratch array (B*H*ceil(L/block)*d*8 bytes must be <= 16 MiB)";
    default: return "unknown error code";
  }
}

const char *blossom_version(void) { return "blossom-gfx950 0.1"; }

}  // extern "C"

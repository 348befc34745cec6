// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once

#include <type_traits>

#include <hip/hip_runtime.h>
#include <stddef.h>

#include "common.h"

// Launches a kernel and leaves the enclosing (void) launcher at once if the launch failed, so that
// no later kernel of a multi-kernel entry point is enqueued on what the failed one should have
// written.  The error stays set for the entry point's final status check.
#define BLOSSOM_LAUNCH(...)                              \
  do {                                                   \
    hipLaunchKernelGGL(__VA_ARGS__);                     \
    if (hipPeekAtLastError() != hipSuccess) return;      \
  } while (0)

namespace blossom {

inline bool launch_failed() { return hipPeekAtLastError() != hipSuccess; }

// Pointers of one forward call (device memory; element type per `dtype`).
struct FwdArgs {
  const void *Q, *K, *V;
  const int *valid_len;
  const int *sel;          // nullptr in dense mode
  const float *gate_w;     // [H,2d]
  const float *gate_b;     // [H] or nullptr
  void *O;
  void *o_lt, *o_st;       // or nullptr
  float *lse_lt, *lse_st;  // or nullptr (dense mode: lse_lt = lse)
  int dense;               // 1: dense causal attention, single branch, no gate
  int kv_groups;           // > 0: `sel` holds one row per query position and key/value group [B,G,L,k], K and V are [B,G,L,d]
};

struct BwdArgs {
  const void *Q, *K, *V;
  const int *valid_len;
  const int *sel;
  const float *gate_w, *gate_b;
  const void *o_lt, *o_st;
  const float *lse_lt, *lse_st;
  const void *dO;
  void *dQ, *dK, *dV;
  float *d_gate_w, *d_gate_b;
  void *ws;
};

// select.hip
size_t select_workspace_bytes(const KParams &p);
// (kcmp: K holds the caller's compressed keys [B,H,NB,d] instead of the keys themselves)
// (p.rope_cos set: the pooling pass rotates Q and K on the way in and writes them to Q_rot, K_rot)
void launch_select(const KParams &p, int dtype, const void *Q, const void *K, bool kcmp, const int *valid_len,
                   int *sel, void *ws, hipStream_t st, void *Q_rot = nullptr, void *K_rot = nullptr);

// Backward workspace, carved from the caller's buffer.
struct BwdWorkspace {
  float4 *rowstat;   // [B*H*L] (alpha, dz, D_lt, D_st)
  int *offs;         // [B*H,(NB+1)] inverse selection list: offsets
  int *items;        // [B*H,NB*k]   inverse selection list: query blocks per key block, in a fixed order;
                     //              bit kInvFewShift marks a query block whose long-term rows may see few keys
  float *partial;    // [B*H*nchunk,(2d+1)] partial gate-weight gradients
  float *stage2;     // [H,slices,(2d+1)] second reduction level
  // matrix-core path only: per-branch upstream gradient dO_x = a_x*dO + dz*Wg_x in bf16, and per
  // row the three-term bf16 splits of (-lse_x*log2(e), -dO_x.o_x) as (hi|mid<<16, lo) pairs
  uint16_t *g_lt, *g_st;      // [B*H*L,d]
  uint4 *rowI_lt, *rowI_st;   // [B*H*L]
  int nchunk;
  size_t total;
};

// Calls f with the head dimension as a compile-time constant (d is one of 8, 16, 32, 64: checked
// at the boundary).
template <typename F>
inline void with_head_dim(int d, F &&f)
{
  switch (d) {
    case 8: f(std::integral_constant<int, 8>{}); break;
    case 16: f(std::integral_constant<int, 16>{}); break;
    case 32: f(std::integral_constant<int, 32>{}); break;
    default: f(std::integral_constant<int, 64>{}); break;
  }
}

// generic.hip: scalar-ALU kernels for every supported (dtype, d, b)
void launch_fwd_generic(const KParams &p, int dtype, const FwdArgs &a, hipStream_t st);
BwdWorkspace bwd_carve(const KParams &p, int dtype, void *ws);
size_t bwd_workspace_bytes(const KParams &p, int dtype);
// inverse selection list entries: query block index, plus a flag for blocks whose selected past
// blocks hold fewer than kInvFewKeys valid keys (their rows carry large probabilities)
constexpr int kInvFewKeys = 32;
constexpr int kInvFewShift = 30;
constexpr int kInvBlockMask = (1 << kInvFewShift) - 1;
enum : unsigned { kBwdStageGate = 1u, kBwdStageInverse = 2u, kBwdStageDQ = 4u, kBwdStageDKV = 8u, kBwdStageAll = 15u };
void launch_bwd(const KParams &p, int dtype, const BwdArgs &a, unsigned stages, hipStream_t st);

// mfma_fwd.hip: matrix-core forward for bf16, d = 64, b in {32, 64}
bool fwd_mfma_supported(const KParams &p, int dtype);
void launch_fwd_mfma(const KParams &p, const FwdArgs &a, hipStream_t st);
// mfma_fwd4.hip: the four-wavefront forward for block size 64 (launch_fwd_mfma dispatches to it)
void launch_fwd_mfma4(const KParams &p, const FwdArgs &a, hipStream_t st);

// mfma_f32.hip: forward, dQ and dK/dV on the fp32 matrix instructions for short sequences (fp32 or bf16
// storage, d in {8, 16, 32}, b in {8, 16}, the streamed tensors of a head resident in LDS)
bool fwd_res_supported(const KParams &p, int dtype);
void launch_fwd_res(const KParams &p, int dtype, const FwdArgs &a, hipStream_t st);
bool fwd_positions_supported(const KParams &p, int dtype);
bool bwd_res_supported(const KParams &p, int dtype);
bool bwd_positions_supported(const KParams &p, int dtype);
void launch_bwd_positions(const KParams &p, int dtype, const BwdArgs &a, const BwdWorkspace &w, int kv_groups, hipStream_t st);
void launch_bwd_res(const KParams &p, int dtype, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st);

// mfma_bwd.hip: matrix-core dQ and dK/dV for bf16, d = 64, b in {32, 64}
bool bwd_mfma_supported(const KParams &p, int dtype);
void launch_bwd_mfma(const KParams &p, const BwdArgs &a, const BwdWorkspace &w, unsigned stages, hipStream_t st);

// out_proj.hip: output projection + residual + LayerNorm around the attention (Eq. 4, the equation after Eq. 19)
struct OutProjArgs {
  int B, H, L, d, Dm, dtype;      // dtype 0 = fp32, 1 = bf16 (O, Wt, Hprev, S)
  const void *O;                  // [B,H,L,d]
  const void *Wt;                 // [Dm, H*d]
  const float *bias;              // [Dm] or nullptr
  const void *Hprev;              // [B,L,Dm]
  const float *gamma, *beta;      // [Dm]
  float eps;
  void *S;                        // [B,L,Dm]
  float *mean, *rstd;             // [B,L] or nullptr
};
bool out_proj_supported(const OutProjArgs &a);
void launch_out_proj(const OutProjArgs &a, hipStream_t st);

}  // namespace blossom

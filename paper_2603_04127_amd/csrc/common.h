// Internal declarations shared by the translation units of the DARK attention library.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_bf16.h>
#include <stddef.h>
#include <stdint.h>

#include "dark.h"

namespace dark {

// ---------------------------------------------------------------------------
// Kernel slots for the optional per-kernel timing (dark_timing_*).
// ---------------------------------------------------------------------------
enum KernelId : int {
  KID_GEMM = 0,        // fp32 batched GEMM of the fp32 path
  KID_LOAD,            // dtype conversion / [V|1] staging
  KID_ROWSTAT,         // logits: subtract norm term, row maxima
  KID_HEADMAX,         // per-head maximum of row maxima
  KID_EXP,             // exponentiation
  KID_SUM_SLICES,      // fixed-order sum of per-slice partial states
  KID_FINISH,          // numerator / denominator
  KID_SCAN,            // exclusive scan of chunk states
  KID_BWD_ELEM,        // element-wise kernels of the backward pass
  KID_PREP,            // fused path: A = sqrt(scale)*log2(e) * W M, operand packing
  KID_KV_REDUCE,       // fused path: phi(K)^T [V|1] per L-slice
  KID_KV_MERGE,        // fused path: fixed-order merge of slice states
  KID_READOUT,         // fused path: phi(Q) S / phi(Q) z
  KID_KEY_NORMS,       // fused causal path: norm term of every key
  KID_CAUSAL_STATE,    // fused causal path: state of every slice
  KID_CAUSAL_PREFIX,   // fused causal path: exclusive prefix over the slice states
  KID_CAUSAL_SCAN,     // fused causal path: tile-by-tile scan inside a slice (inter + intra term)
  KID_FEATURIZE,       // fused path: feature map written to memory (dark_featurize)
  KID_BWD_FWD,         // fused backward: forward-order pass (denominators, dQ, query half of dA, suffix-state pieces)
  KID_BWD_SUFFIX,      // fused backward: exclusive suffix sums of the slices' reverse-state pieces
  KID_BWD_REV,         // fused backward: reverse-order pass (dV, dK, key half of dA, norm-term matrix)
  KID_BWD_DM,          // fused backward: sums over slices and dM per head
  KID_WHITEN_MOMENTS,  // whitening geometry: second moments of the rows of Q and K
  KID_WHITEN_EIG,      // whitening geometry: eigen-decomposition, M = Lambda^-1/2
  KID_DECODE,          // one-token recurrence of causal attention
  KID_COUNT
};

const char* kernel_name(int k);
bool timing_on();
// A pair of events for one launch: hipExtLaunchKernelGGL stamps them with the kernel's own begin and end
// on the device, so their difference is the kernel's duration without the launch gap around it.  The
// stream is drained first: a dispatch queued behind running work is stamped when it is picked up, not
// when its first wave starts.
void timing_events(int kid, hipStream_t st, hipEvent_t* start, hipEvent_t* stop);

// Launch helper: optional per-kernel timing, launch-error check.
#define DARK_LAUNCH(kid, st, kernel, grid, block, shmem, ...)                                       \
  do {                                                                                              \
    if (::dark::timing_on()) {                                                                      \
      hipEvent_t _ea, _eb;                                                                          \
      ::dark::timing_events((kid), (st), &_ea, &_eb);                                                  \
      hipExtLaunchKernelGGL(kernel, (grid), (block), (shmem), (st), _ea, _eb, 0, __VA_ARGS__);      \
    } else {                                                                                        \
      hipLaunchKernelGGL(kernel, (grid), (block), (shmem), (st), __VA_ARGS__);                      \
    }                                                                                               \
    if (hipGetLastError() != hipSuccess) return DARK_EHIP;                                          \
  } while (0)

#define DARK_TRY(expr)                       \
  do {                                       \
    dark_status _s = (expr);                 \
    if (_s != DARK_OK) return _s;            \
  } while (0)

// ---------------------------------------------------------------------------
// Bump allocator over the caller's workspace.  With base == nullptr it only
// measures (used by dark_workspace_bytes).
// ---------------------------------------------------------------------------
struct Arena {
  char* base;
  size_t cap;
  size_t off;
  bool overflow;
  Arena(void* b, size_t c) : base(static_cast<char*>(b)), cap(c), off(0), overflow(false) {}
  template <typename T>
  T* take(size_t n) {
    size_t bytes = (n * sizeof(T) + 255) & ~size_t(255);
    size_t at = off;
    off += bytes;
    if (base == nullptr) return nullptr;
    if (off > cap) {
      overflow = true;
      return nullptr;
    }
    return reinterpret_cast<T*>(base + at);
  }
};

struct Problem {
  dark_params p;
  float scale;     // resolved (never 0)
  int chunk;       // resolved
  bool m_identity = false;  // the caller passed M == NULL: Sigma = I (needs r == d)
  // Hand-over of the causal forward's operand copies, key norms and prefix states to the backward:
  // 0 = none, 1 = the forward writes them into `saved`, 2 = the backward reads them from `saved`.
  int saved_mode = 0;
  void* saved = nullptr;
  size_t saved_bytes = 0;
  hipStream_t st;
  long long BH() const { return (long long)p.B * p.H; }
  long long rows() const { return (long long)p.B * p.H * p.L; }
};

// Parameter validation shared by all entry points (no HIP call).
dark_status check_params(const dark_params* p, Problem* out);
inline bool aligned(const void* q, size_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) == 0; }

// M[h] = I for every head, into a [H, d, d] fp32 buffer (generic.hip).
dark_status fill_identity(const Problem& pb, float* Mid);
// fp32 path (generic.hip).  With arena.base == nullptr these only measure.
dark_status f32_featurize(const Problem& pb, Arena& ar, const void* X, const float* M, const float* W,
                          int is_query, void* phi, float* stab);
dark_status f32_attn_fwd(const Problem& pb, Arena& ar, bool causal, const void* Q, const void* K,
                         const void* V, const float* M, const float* W, void* out);
dark_status f32_attn_bwd(const Problem& pb, Arena& ar, bool causal, const void* Q, const void* K,
                         const void* V, const float* M, const float* W, const void* dOut, float* dQ,
                         float* dK, float* dV, float* dM, float* dW);
// dW[h][j][t] = alpha sum over the nb batch entries b and over c of T[b][h][j][c] M[h][t][c]  (T: [nb, H, m, d]);
// with a shared W the heads are summed as well (generic.hip).
dark_status launch_dw(const Problem& pb, const float* T, int nb, const float* M, float* dW);

// Bytes of the hand-over buffer of the causal forward/backward pair on the MFMA path (0: no hand-over for
// these parameters).  fused_causal.hip.
size_t fused_saved_causal_bytes(const Problem& pb);
// One-token causal recurrence (decode.hip).
dark_status decode_step(const Problem& pb, const void* q, const void* k, const void* v, const float* M,
                        const float* W, float* S, float* z, float* c, void* out);
// Whitening geometry (whiten.hip).  With arena.base == nullptr it only measures.
bool whiten_supported(const Problem& pb);
dark_status whiten(const Problem& pb, Arena& ar, const void* Q, const void* K, float* M, float* cov_out);
// fused MFMA feature map (fused_feat.hip).
bool fused_featurize_supported(const Problem& pb);
dark_status fused_featurize(const Problem& pb, Arena& ar, const void* X, const float* M, const float* W,
                            int is_query, void* phi, float* stab);

// fused MFMA path (fused.hip).
bool fused_supported(const Problem& pb, int op, bool causal);
dark_status fused_attn_fwd(const Problem& pb, Arena& ar, const void* Q, const void* K, const void* V,
                           const float* M, const float* W, void* out);
dark_status fused_attn_causal_fwd(const Problem& pb, Arena& ar, const void* Q, const void* K,
                                  const void* V, const float* M, const float* W, void* out);

// fused MFMA backward (fused_bwd.hip): causal, bf16, d = r = dv = 64, m = 256.
bool fused_bwd_supported(const Problem& pb, bool causal);
dark_status fused_attn_bwd(const Problem& pb, Arena& ar, const void* Q, const void* K, const void* V,
                           const float* M, const float* W, const void* dOut, float* dQ, float* dK,
                           float* dV, float* dM, float* dW);

}  // namespace dark

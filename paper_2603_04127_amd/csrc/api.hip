// C-ABI entry points of the DARK attention library: argument checks, path
// selection and the optional per-kernel timing.  No kernel lives here.
#include <cmath>
#include <vector>

#include "common.h"

namespace dark {

// ---------------------------------------------------------------------------
// timing
// ---------------------------------------------------------------------------
namespace {
struct Pending {
  int kid;
  hipEvent_t a, b;
};
bool g_timing = false;
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_free;
double g_total_ms[KID_COUNT];
int64_t g_launches[KID_COUNT];

hipEvent_t get_event() {
  if (!g_free.empty()) {
    hipEvent_t e = g_free.back();
    g_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}
}  // namespace

const char* kernel_name(int k) {
  static const char* names[KID_COUNT] = {
      "f32_gemm",     "f32_load",   "f32_rowstat",  "f32_headmax",  "f32_exp",      "f32_sum_slices",
      "f32_finish",   "f32_scan",   "f32_bwd_elem", "fused_prep",   "fused_kv_reduce", "fused_kv_merge",
      "fused_readout", "fused_key_norms", "fused_causal_state", "fused_causal_prefix", "fused_causal_scan", "fused_featurize",
      "fused_bwd_fwd", "fused_bwd_suffix", "fused_bwd_rev", "fused_bwd_dm", "whiten_moments", "whiten_eig", "decode_step"};
  return (k >= 0 && k < KID_COUNT) ? names[k] : "?";
}
bool timing_on() { return g_timing; }
void timing_events(int kid, hipStream_t st, hipEvent_t* start, hipEvent_t* stop) {
  (void)hipStreamSynchronize(st);
  *start = get_event();
  *stop = get_event();
  g_pending.push_back({kid, *start, *stop});
}

static void drain() {
  for (auto& pd : g_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(pd.b) == hipSuccess && hipEventElapsedTime(&ms, pd.a, pd.b) == hipSuccess) {
      g_total_ms[pd.kid] += ms;
      g_launches[pd.kid] += 1;
    }
    g_free.push_back(pd.a);
    g_free.push_back(pd.b);
  }
  g_pending.clear();
}

// ---------------------------------------------------------------------------
// validation
// ---------------------------------------------------------------------------
dark_status check_params(const dark_params* p, Problem* out) {
  if (p == nullptr) return DARK_EINVAL;
  if (p->B < 0 || p->L < 0) return DARK_EINVAL;
  if (p->H <= 0 || p->d <= 0 || p->r <= 0 || p->m <= 0 || p->dv <= 0) return DARK_EINVAL;
  if (p->chunk < 0) return DARK_EINVAL;
  if (p->io_dtype != DARK_F32 && p->io_dtype != DARK_BF16) return DARK_EINVAL;
  if (p->out_dtype != DARK_F32 && p->out_dtype != DARK_BF16) return DARK_EINVAL;
  if (p->path != DARK_PATH_AUTO && p->path != DARK_PATH_F32 && p->path != DARK_PATH_FUSED) return DARK_EINVAL;
  if (!(p->scale >= 0.f) || std::isinf(p->scale)) return DARK_EINVAL;
  if (p->sched_kv_wgs < 0 || p->sched_ro_wgs < 0 || p->sched_cs_wgs < 0 || p->sched_cs_state < 0) return DARK_EINVAL;
  // Index arithmetic is 64-bit, but single dimensions must stay well inside int32.
  if ((long long)p->L * p->m > (1LL << 40) || p->d > 65536 || p->m > (1 << 20) || p->dv > 65536 || p->r > 65536)
    return DARK_EUNSUPPORTED;
  out->p = *p;
  out->scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->d);
  out->chunk = p->chunk > 0 ? p->chunk : 128;
  if (out->chunk > 1024) return DARK_EUNSUPPORTED;
  out->st = nullptr;
  return DARK_OK;
}

static dark_status check_ws(const void* ws, size_t ws_bytes, size_t need) {
  if (need == 0) return DARK_OK;
  if (ws == nullptr || ws_bytes < need) return DARK_EWORKSPACE;
  if (!aligned(ws, 256)) return DARK_EALIGN;
  return DARK_OK;
}

static bool use_fused(const Problem& pb, int op, bool causal, dark_status* err) {
  *err = DARK_OK;
  if (pb.p.path == DARK_PATH_F32) return false;
  bool ok = op == DARK_OP_FEATURIZE ? fused_featurize_supported(pb)
            : op == DARK_OP_ATTN_BWD ? fused_bwd_supported(pb, causal)
                                     : fused_supported(pb, op, causal);
  if (!ok && pb.p.path == DARK_PATH_FUSED) *err = DARK_EUNSUPPORTED;
  return ok;
}

static dark_status run(const Problem& pb, Arena& ar, int op, bool causal, const void* Q, const void* K,
                       const void* V, const float* M, const float* W, const void* dOut, void* out,
                       float* stab, int is_query, float* dQ, float* dK, float* dV, float* dM,
                       float* dW = nullptr) {
  dark_status err;
  bool fused = use_fused(pb, op, causal, &err);
  if (err != DARK_OK) return err;
  // M == NULL stands for the identity (isotropic positive random features): it is written out here, so that
  // every kernel downstream sees an ordinary M.  The buffer is part of every plan with r == d.
  if (pb.p.r == pb.p.d) {
    float* Mid = ar.take<float>((size_t)pb.p.H * pb.p.d * pb.p.d);
    if (pb.m_identity && ar.base != nullptr && !ar.overflow) {
      DARK_TRY(fill_identity(pb, Mid));
      M = Mid;
    }
  }
  switch (op) {
    case DARK_OP_FEATURIZE:
      return fused ? fused_featurize(pb, ar, Q, M, W, is_query, out, stab)
                   : f32_featurize(pb, ar, Q, M, W, is_query, out, stab);
    case DARK_OP_ATTN_FWD:
      return fused ? fused_attn_fwd(pb, ar, Q, K, V, M, W, out) : f32_attn_fwd(pb, ar, false, Q, K, V, M, W, out);
    case DARK_OP_ATTN_CAUSAL_FWD:
      return fused ? fused_attn_causal_fwd(pb, ar, Q, K, V, M, W, out)
                   : f32_attn_fwd(pb, ar, true, Q, K, V, M, W, out);
    case DARK_OP_ATTN_BWD:
      return fused ? fused_attn_bwd(pb, ar, Q, K, V, M, W, dOut, dQ, dK, dV, dM, dW)
                   : f32_attn_bwd(pb, ar, causal, Q, K, V, M, W, dOut, dQ, dK, dV, dM, dW);
  }
  return DARK_EINVAL;
}

// ---------------------------------------------------------------------------
// Scratch of the entry point that allocates nothing (dark_attn_fwd_static): a fixed
// array in device memory, one copy per GPU.  In host code the array's name is only a
// stand-in: its device address is asked for once per device and kept.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = DARK_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];

static dark_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DARK_EHIP;
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return DARK_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DARK_OK;
}

static size_t measure(const Problem& pb, int op, bool causal) {
  Arena ar(nullptr, 0);
  // In measuring mode the paths only walk their allocation plan; pointers are unused.
  dark_status s = run(pb, ar, op, causal, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1,
                      (float*)1, (float*)1, (float*)1, (float*)1);
  if (s != DARK_OK) return 0;
  return ar.off;
}

}  // namespace dark

using namespace dark;

extern "C" {

int dark_version(void) { return 100; }

const char* dark_status_string(dark_status s) {
  switch (s) {
    case DARK_OK: return "ok";
    case DARK_EINVAL: return "invalid argument";
    case DARK_EUNSUPPORTED: return "unsupported shape or dtype for the requested path";
    case DARK_EWORKSPACE: return "workspace missing or too small";
    case DARK_EALIGN: return "misaligned pointer";
    case DARK_EHIP: return "HIP runtime error";
    case DARK_ESCRATCH: return "problem needs more scratch than the static buffer of dark_attn_fwd_static holds";
  }
  return "unknown status";
}

size_t dark_workspace_bytes(const dark_params* p, int op, int causal) {
  Problem pb;
  if (check_params(p, &pb) != DARK_OK) return 0;
  if (op < DARK_OP_FEATURIZE || op > DARK_OP_WHITEN) return 0;
  if (pb.p.B == 0 || pb.p.L == 0) return 0;
  if (op == DARK_OP_WHITEN) {
    if (!whiten_supported(pb)) return 0;
    Arena ar(nullptr, 0);
    (void)whiten(pb, ar, nullptr, nullptr, nullptr, nullptr);
    return ar.off;
  }
  return measure(pb, op, causal != 0 || op == DARK_OP_ATTN_CAUSAL_FWD);
}

dark_status dark_featurize(const dark_params* p, const void* X, const float* M, const float* W, int is_query,
                           void* phi, float* stab, void* ws, size_t ws_bytes, void* hip_stream) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (pb.p.B == 0 || pb.p.L == 0) return DARK_OK;
  if (X == nullptr || W == nullptr || phi == nullptr) return DARK_EINVAL;
  if (M == nullptr && pb.p.r != pb.p.d) return DARK_EINVAL;  // M == NULL: identity, needs r == d
  pb.m_identity = M == nullptr;
  if (!aligned(X, 16) || !aligned(M, 16) || !aligned(W, 16) || !aligned(phi, 16) || !aligned(stab, 4))
    return DARK_EALIGN;
  {
    dark_status err;
    (void)use_fused(pb, DARK_OP_FEATURIZE, false, &err);
    if (err != DARK_OK) return err;
  }
  DARK_TRY(check_ws(ws, ws_bytes, measure(pb, DARK_OP_FEATURIZE, false)));
  pb.st = static_cast<hipStream_t>(hip_stream);
  Arena ar(ws, ws_bytes);
  return run(pb, ar, DARK_OP_FEATURIZE, false, X, nullptr, nullptr, M, W, nullptr, phi, stab, is_query, nullptr,
             nullptr, nullptr, nullptr);
}

// Validates a hand-over buffer and arms the problem with it (mode 1: the forward writes, 2: the backward reads).
// Parameters without a hand-over (dark_saved_bytes() == 0) ignore the buffer.
static dark_status arm_saved(Problem& pb, int mode, void* saved, size_t saved_bytes) {
  const size_t need = fused_saved_causal_bytes(pb);
  if (need == 0) return DARK_OK;
  if (saved == nullptr || saved_bytes < need) return DARK_EWORKSPACE;
  if (!aligned(saved, 256)) return DARK_EALIGN;
  pb.saved_mode = mode;
  pb.saved = saved;
  pb.saved_bytes = saved_bytes;
  return DARK_OK;
}

static dark_status attn_common(const dark_params* p, int op, const void* Q, const void* K, const void* V,
                               const float* M, const float* W, void* out, void* ws, size_t ws_bytes,
                               void* hip_stream, void* saved = nullptr, size_t saved_bytes = 0, bool save = false) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (save) DARK_TRY(arm_saved(pb, 1, saved, saved_bytes));
  if (pb.p.B == 0 || pb.p.L == 0) return DARK_OK;
  if (!Q || !K || !V || !W || !out) return DARK_EINVAL;
  if (M == nullptr && pb.p.r != pb.p.d) return DARK_EINVAL;  // M == NULL: identity, needs r == d
  pb.m_identity = M == nullptr;
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(M, 16) || !aligned(W, 16) ||
      !aligned(out, 16))
    return DARK_EALIGN;
  bool causal = op == DARK_OP_ATTN_CAUSAL_FWD;
  dark_status err;
  (void)use_fused(pb, op, causal, &err);
  if (err != DARK_OK) return err;
  DARK_TRY(check_ws(ws, ws_bytes, measure(pb, op, causal)));
  pb.st = static_cast<hipStream_t>(hip_stream);
  Arena ar(ws, ws_bytes);
  return run(pb, ar, op, causal, Q, K, V, M, W, nullptr, out, nullptr, 0, nullptr, nullptr, nullptr, nullptr);
}

dark_status dark_attn_fwd(const dark_params* p, const void* Q, const void* K, const void* V, const float* M,
                          const float* W, void* out, void* ws, size_t ws_bytes, void* hip_stream) {
  return attn_common(p, DARK_OP_ATTN_FWD, Q, K, V, M, W, out, ws, ws_bytes, hip_stream);
}

size_t dark_static_scratch_bytes(void) { return kStaticScratchBytes; }

dark_status dark_attn_fwd_static(const dark_params* p, const void* Q, const void* K, const void* V, const float* M,
                                 const float* W, void* out, void* hip_stream) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (pb.p.B == 0 || pb.p.L == 0) return DARK_OK;
  if (!Q || !K || !V || !W || !out) return DARK_EINVAL;
  if (M == nullptr && pb.p.r != pb.p.d) return DARK_EINVAL;  // M == NULL: identity, needs r == d
  pb.m_identity = M == nullptr;
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(M, 16) || !aligned(W, 16) ||
      !aligned(out, 16))
    return DARK_EALIGN;
  dark_status err;
  (void)use_fused(pb, DARK_OP_ATTN_FWD, false, &err);
  if (err != DARK_OK) return err;
  if (measure(pb, DARK_OP_ATTN_FWD, false) > kStaticScratchBytes) return DARK_ESCRATCH;  // before any HIP call
  void* ws = nullptr;
  DARK_TRY(static_scratch(&ws));
  pb.st = static_cast<hipStream_t>(hip_stream);
  Arena ar(ws, kStaticScratchBytes);
  return run(pb, ar, DARK_OP_ATTN_FWD, false, Q, K, V, M, W, nullptr, out, nullptr, 0, nullptr, nullptr, nullptr,
             nullptr);
}

dark_status dark_attn_causal_fwd(const dark_params* p, const void* Q, const void* K, const void* V,
                                 const float* M, const float* W, void* out, void* ws, size_t ws_bytes,
                                 void* hip_stream) {
  return attn_common(p, DARK_OP_ATTN_CAUSAL_FWD, Q, K, V, M, W, out, ws, ws_bytes, hip_stream);
}

dark_status dark_whiten(const dark_params* p, const void* Q, const void* K, float* M_out, float* cov_out, void* ws,
                        size_t ws_bytes, void* hip_stream) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (pb.p.B == 0 || pb.p.L == 0) return DARK_EINVAL;  // no rows, no covariance
  if (Q == nullptr || M_out == nullptr) return DARK_EINVAL;
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(M_out, 16) || !aligned(cov_out, 16)) return DARK_EALIGN;
  if (!whiten_supported(pb)) return DARK_EUNSUPPORTED;
  Arena measure_ar(nullptr, 0);
  (void)whiten(pb, measure_ar, nullptr, nullptr, nullptr, nullptr);
  DARK_TRY(check_ws(ws, ws_bytes, measure_ar.off));
  pb.st = static_cast<hipStream_t>(hip_stream);
  Arena ar(ws, ws_bytes);
  return whiten(pb, ar, Q, K, M_out, cov_out);
}

dark_status dark_decode_step(const dark_params* p, const void* q, const void* k, const void* v, const float* M,
                             const float* W, float* S, float* z, float* c, void* out, void* hip_stream) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (pb.p.B == 0) return DARK_OK;
  if (!q || !k || !v || !W || !S || !z || !c || !out) return DARK_EINVAL;
  if (M == nullptr && pb.p.r != pb.p.d) return DARK_EINVAL;  // M == NULL: identity, needs r == d
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(M, 16) || !aligned(W, 16) || !aligned(S, 16) ||
      !aligned(z, 16) || !aligned(c, 4) || !aligned(out, 16))
    return DARK_EALIGN;
  pb.st = static_cast<hipStream_t>(hip_stream);
  return decode_step(pb, q, k, v, M, W, S, z, c, out);
}

size_t dark_saved_bytes(const dark_params* p) {
  Problem pb;
  if (check_params(p, &pb) != DARK_OK) return 0;
  if (pb.p.B == 0 || pb.p.L == 0) return 0;
  return fused_saved_causal_bytes(pb);
}

dark_status dark_attn_causal_fwd_save(const dark_params* p, const void* Q, const void* K, const void* V,
                                      const float* M, const float* W, void* out, void* saved, size_t saved_bytes,
                                      void* ws, size_t ws_bytes, void* hip_stream) {
  return attn_common(p, DARK_OP_ATTN_CAUSAL_FWD, Q, K, V, M, W, out, ws, ws_bytes, hip_stream, saved, saved_bytes, true);
}

}  // extern "C"

static dark_status bwd_common(const dark_params* p, int causal, const void* Q, const void* K, const void* V,
                              const float* M, const float* W, const void* dOut, float* dQ, float* dK, float* dV,
                              float* dM, float* dW, void* ws, size_t ws_bytes, void* hip_stream, const void* saved,
                              size_t saved_bytes, bool use_saved) {
  Problem pb;
  DARK_TRY(check_params(p, &pb));
  if (use_saved) DARK_TRY(arm_saved(pb, 2, const_cast<void*>(saved), saved_bytes));
  if (pb.p.B == 0 || pb.p.L == 0) return DARK_OK;  // nothing to enqueue; gradients are left untouched
  if (!Q || !K || !V || !W || !dOut) return DARK_EINVAL;
  if (M == nullptr && pb.p.r != pb.p.d) return DARK_EINVAL;  // M == NULL: identity, needs r == d
  pb.m_identity = M == nullptr;
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(M, 16) || !aligned(W, 16) ||
      !aligned(dOut, 16) || !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16) || !aligned(dM, 16) || !aligned(dW, 16))
    return DARK_EALIGN;
  {
    dark_status err;
    (void)use_fused(pb, DARK_OP_ATTN_BWD, causal != 0, &err);
    if (err != DARK_OK) return err;
  }
  DARK_TRY(check_ws(ws, ws_bytes, measure(pb, DARK_OP_ATTN_BWD, causal != 0)));
  pb.st = static_cast<hipStream_t>(hip_stream);
  Arena ar(ws, ws_bytes);
  return run(pb, ar, DARK_OP_ATTN_BWD, causal != 0, Q, K, V, M, W, dOut, nullptr, nullptr, 0, dQ, dK, dV, dM, dW);
}

extern "C" {

dark_status dark_attn_bwd_dw(const dark_params* p, int causal, const void* Q, const void* K, const void* V,
                             const float* M, const float* W, const void* dOut, float* dQ, float* dK, float* dV,
                             float* dM, float* dW, void* ws, size_t ws_bytes, void* hip_stream) {
  return bwd_common(p, causal, Q, K, V, M, W, dOut, dQ, dK, dV, dM, dW, ws, ws_bytes, hip_stream, nullptr, 0, false);
}

dark_status dark_attn_bwd_saved(const dark_params* p, const void* Q, const void* K, const void* V, const float* M,
                                const float* W, const void* dOut, const void* saved, size_t saved_bytes, float* dQ,
                                float* dK, float* dV, float* dM, float* dW, void* ws, size_t ws_bytes,
                                void* hip_stream) {
  return bwd_common(p, 1, Q, K, V, M, W, dOut, dQ, dK, dV, dM, dW, ws, ws_bytes, hip_stream, saved, saved_bytes, true);
}

dark_status dark_attn_bwd(const dark_params* p, int causal, const void* Q, const void* K, const void* V,
                          const float* M, const float* W, const void* dOut, float* dQ, float* dK, float* dV,
                          float* dM, void* ws, size_t ws_bytes, void* hip_stream) {
  return dark_attn_bwd_dw(p, causal, Q, K, V, M, W, dOut, dQ, dK, dV, dM, nullptr, ws, ws_bytes, hip_stream);
}

void dark_timing_enable(int on) { g_timing = on != 0; }

void dark_timing_reset(void) {
  drain();
  for (int k = 0; k < KID_COUNT; ++k) {
    g_total_ms[k] = 0.0;
    g_launches[k] = 0;
  }
}

int dark_timing_slots(void) { return KID_COUNT; }

dark_status dark_timing_read(int k, const char** name, int64_t* launches, double* total_ms) {
  if (k < 0 || k >= KID_COUNT) return DARK_EINVAL;
  drain();
  if (name) *name = kernel_name(k);
  if (launches) *launches = g_launches[k];
  if (total_ms) *total_ms = g_total_ms[k];
  return DARK_OK;
}

}  // extern "C"

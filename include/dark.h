/*
 * dark.h - C ABI of the DARK attention library for AMD MI355X (gfx950).
 *
 * The library computes the positive-random-feature estimator of the data-aligned
 * softmax kernel exp(q^T Sigma k / sqrt(d)), Sigma = M^T M (paper: Section 4.1,
 * Eq. (3)), and the linear-time attention built on it (paper: Section 2,
 * "Efficient attention via random feature kernels").
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every data pointer is DEVICE memory owned by the caller, 16-byte aligned,
 *    contiguous, row-major with the last listed index fastest.  The library never
 *    allocates, frees or synchronises: it enqueues kernels on `hip_stream`
 *    (a hipStream_t passed as void*, NULL = the default stream) and returns.
 *    Scratch memory comes from the caller (`ws`, at least
 *    dark_workspace_bytes() bytes, 256-byte aligned).  Calls that share a
 *    workspace must be ordered on one stream.
 *  - Q, K: [B, H, L, d];  V: [B, H, L, dv];  M: [H, r, d] (shared over the batch);
 *    W: [H, m, r], or [m, r] when w_shared != 0.  M and W are always float32.
 *    M may be NULL in every entry point: it then stands for the identity (Sigma = I, the
 *    isotropic positive random features of Section 2, Eq. (1), which the paper compares
 *    against in Section 6) and r must equal d (else DARK_EINVAL).  The identity is written
 *    into the workspace and the same kernels run; only the key-norm kernel of the causal
 *    MFMA path at d = 128 takes a shorter route (|k|^2 without a projection).  dM of
 *    dark_attn_bwd is then the gradient at M = I.
 *    Q, K, V, dOut, phi and out have the element type `io_dtype`
 *    (out: `out_dtype`); gradients are always float32.
 *  - Each query and key is multiplied by sqrt(scale) before the feature map, so
 *    the estimated kernel is exp(scale * q^T Sigma k); scale == 0 selects
 *    1/sqrt(d) (paper: Section 2, footnote on absorbing the 1/sqrt(d) scaling).
 *  - No epsilon is added anywhere.  Stabilising shifts inside the exponentials
 *    cancel exactly in every attention output.
 *  - Return value: DARK_OK, or an error code.  All argument checks happen before
 *    the first HIP call, so they can be exercised without a GPU.  On error the
 *    outputs are undefined.  Results are run-to-run bitwise deterministic (no
 *    floating-point atomics).
 *  - B == 0 or L == 0 is a valid empty problem: nothing is enqueued, DARK_OK.
 */
#ifndef DARK_H_
#define DARK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DARK_OK = 0,
  DARK_EINVAL = 1,       /* null pointer, non-positive dimension, bad enum value */
  DARK_EUNSUPPORTED = 2, /* shape / dtype not supported by the requested path */
  DARK_EWORKSPACE = 3,   /* ws == NULL or ws_bytes too small */
  DARK_EALIGN = 4,       /* a pointer is not 16-byte aligned (ws: 256) */
  DARK_EHIP = 5,         /* a HIP runtime call failed (launch error) */
  DARK_ESCRATCH = 6      /* dark_attn_fwd_static: the problem needs more than the static scratch */
} dark_status;

typedef enum { DARK_F32 = 0, DARK_BF16 = 1 } dark_dtype;

typedef enum {
  DARK_OP_FEATURIZE = 0,
  DARK_OP_ATTN_FWD = 1,
  DARK_OP_ATTN_CAUSAL_FWD = 2,
  DARK_OP_ATTN_BWD = 3,
  DARK_OP_WHITEN = 4
} dark_op;

/*
 * Numerical range of the two families of kernels.
 *
 * Fused MFMA kernels, what DARK_PATH_AUTO takes for bf16 io with d = r = dv in {64, 128} and m = 256
 * (bidirectional forward also m = 512 at d = 64; dark_featurize any m that is a multiple of 64 and fits the
 * LDS; backward only causal, d = 64, m = 256): rows of Q, K (and X of dark_featurize) are converted
 * bf16 -> fp16 and projected by fp16 MFMAs with fp32 accumulation.
 *   - Elements of magnitude in [2^-14, 65504] convert exactly; smaller ones lose bits (absolute error at
 *     most 2^-25 per element); larger ones have no fp16 value and become +-infinity: every output row that
 *     depends on such an element is then non-finite (NaN), never the result of a clamped input.
 *   - A key whose norm term (log2(e)/2) |sqrt(scale) M k|^2 exceeds 65504 contributes features that are
 *     zero to within fp32; it is treated as exactly that (no clamped norm enters).
 *   - The projection operands are rounded to fp16, so a logit w.x~ carries an error of about 2^-11 |w.x~|:
 *     the tolerance quoted for the bf16 path holds for |w.x~| up to a few hundred.
 *   - Stabilisers: one shift per (b, h) and block of 64 features (bidirectional; the readout adds a running
 *     shift per row when a row's logits leave the fp32 exponent range), one scalar shift per slice of a
 *     sequence, the running maximum along it (causal forward and backward: key logits may rise or fall along
 *     a sequence without limit).  Keys more than about 80 nats (2^115) below the shift they are stored under
 *     vanish; a row all of whose keys have vanished comes out non-finite (0/0).
 * fp32 kernels (DARK_PATH_F32; any shape and dtype): inputs of any finite magnitude; bidirectional attention
 * keeps a shift per feature and per row and has no range limit; the causal passes (forward and backward)
 * keep the per-feature shifts per chunk, as running maxima along the sequence, and rescale the chunk states
 * where they are added up: key logits may rise or fall along a sequence without limit, and what has to stay
 * within about 80 nats is the spread of a feature's key logits inside one chunk (p->chunk positions, the
 * keys after the query included).
 * None of these conditions is checked on the host: the entry points only enqueue work.
 */
typedef enum {
  DARK_PATH_AUTO = 0,   /* fused MFMA kernels when the shape allows, else the fp32 kernels */
  DARK_PATH_F32 = 1,    /* fp32 arithmetic throughout (any shape, any io_dtype) */
  DARK_PATH_FUSED = 2   /* fused MFMA kernels or DARK_EUNSUPPORTED */
} dark_path;

typedef struct {
  int32_t B, H, L;   /* batch, heads, sequence length */
  int32_t d;         /* query/key dimension */
  int32_t r;         /* rows of M (r <= d in the paper; any r >= 1 accepted) */
  int32_t m;         /* number of random features */
  int32_t dv;        /* value dimension */
  int32_t chunk;     /* causal chunk length, 0 = 128; a schedule, not semantics */
  int32_t io_dtype;  /* dark_dtype of Q, K, V, dOut, phi */
  int32_t out_dtype; /* dark_dtype of out */
  float scale;       /* 0 = 1/sqrt(d) */
  int32_t w_shared;  /* W is [m, r] for all heads */
  int32_t path;      /* dark_path */
  /* Schedule overrides of the fused MFMA kernels, for tests and tuning; 0 = the library's choice.
   * They change how many slices a sequence is cut into, hence dark_workspace_bytes(), the order of
   * summation and with it the low bits of the result (never the mathematics).  Negative: DARK_EINVAL. */
  int32_t sched_kv_wgs;   /* bidirectional key/value pass: workgroups to aim for (default 512; 256 at d = 128) */
  int32_t sched_ro_wgs;   /* bidirectional readout: workgroups to aim for (default 256) */
  int32_t sched_cs_wgs;   /* causal pass: workgroups (slices over all (b,h)) to aim for (default 256) */
  int32_t sched_cs_state; /* causal pass at d = 64: 1 = slice states by the 8-wave state kernel, else the key/value pass */
} dark_params;

/* Library version (major*10000 + minor*100 + patch). */
int dark_version(void);

/* Human-readable name of a status code (static storage). */
const char* dark_status_string(dark_status s);

/*
 * Bytes of scratch the given operation needs for these parameters on the path the
 * library would choose (0 on invalid parameters).  `op` is a dark_op; for
 * DARK_OP_ATTN_BWD the causal flag is taken from `causal`.
 */
size_t dark_workspace_bytes(const dark_params* p, int op, int causal);

/*
 * Feature map phi_Sigma (paper: Section 4.1, definition before Eq. (3)), with
 * omega~_j = M^T w_j (Appendix B, derivation of Eq. (3)).  For every row x of X
 * [B, H, L, d]:   x' = sqrt(scale) x,  logit_j = w_j^T (M x') - 1/2 ||M x'||^2,
 *                 phi_j = exp(logit_j - c) / sqrt(m).
 * is_query != 0: c is the maximum logit of the row, stab is [B, H, L];
 * is_query == 0: c is the maximum logit over the whole (b, h) slice, stab is [B, H].
 * phi: [B, H, L, m] in io_dtype.  stab (float32) receives c; phi * exp(c) is the
 * unstabilised feature vector.  stab may be NULL.
 */
dark_status dark_featurize(const dark_params* p, const void* X, const float* M, const float* W,
                           int is_query, void* phi, float* stab,
                           void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Bidirectional random-feature attention (paper: Section 2, "Efficient attention
 * via random feature kernels", with the normalisation of the footnote there):
 *   S = phi(K)^T V,  z = phi(K)^T 1,  out_i = phi(q_i)^T S / phi(q_i)^T z
 * per (b, h), with phi as in dark_featurize.  out: [B, H, L, dv] in out_dtype.
 */
dark_status dark_attn_fwd(const dark_params* p, const void* Q, const void* K, const void* V,
                          const float* M, const float* W, void* out,
                          void* ws, size_t ws_bytes, void* hip_stream);

/*
 * dark_attn_fwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bitwise the same result as
 * dark_attn_fwd, minus `ws`: the scratch is a fixed array of
 * DARK_STATIC_SCRATCH_BYTES in device memory that every GPU the library runs on
 * holds until the process ends.  The call allocates and frees nothing.  A problem
 * whose dark_workspace_bytes(p, DARK_OP_ATTN_FWD, 0) exceeds
 * dark_static_scratch_bytes() is rejected with DARK_ESCRATCH before any HIP call.
 * All calls on one GPU share that GPU's array, which keeps the last call's
 * contents (every part that is read is written first by the same call): calls
 * that overlap on one GPU (two streams, two threads) race; order them.
 */
#define DARK_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
size_t dark_static_scratch_bytes(void);
dark_status dark_attn_fwd_static(const dark_params* p, const void* Q, const void* K, const void* V,
                                 const float* M, const float* W, void* out, void* hip_stream);

/*
 * Causal form: out_i uses only keys l <= i (prefix sums of S and z).  The
 * fp32 kernels process the sequence in chunks of p->chunk positions, the fused
 * MFMA kernels in slices and tiles of their own choosing; the result does not
 * depend on either, and L need not be a multiple of anything.
 * Same arguments as dark_attn_fwd.
 */
dark_status dark_attn_causal_fwd(const dark_params* p, const void* Q, const void* K, const void* V,
                                 const float* M, const float* W, void* out,
                                 void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Gradients of sum(out * dOut) for dark_attn_fwd (causal == 0) or
 * dark_attn_causal_fwd (causal != 0).  The paper makes M learnable (Section 4,
 * Sigma = M^T M is learned); the gradients are the chain rule through the
 * definitions above, with W held fixed.
 *   dQ, dK: [B, H, L, d], dV: [B, H, L, dv], float32, overwritten.
 *   dM: [H, r, d], float32, overwritten with the sum over the batch of both the
 *   query-side and the key-side contributions.  Any of dQ, dK, dV, dM may be NULL
 *   (that gradient is skipped).
 * The forward quantities are recomputed; no saved activations are needed.
 */
dark_status dark_attn_bwd(const dark_params* p, int causal, const void* Q, const void* K,
                          const void* V, const float* M, const float* W, const void* dOut,
                          float* dQ, float* dK, float* dV, float* dM,
                          void* ws, size_t ws_bytes, void* hip_stream);

/*
 * dark_attn_bwd with one more output: the gradient with respect to the draws W, which turns
 * the kernel into the learned feature kernel the paper compares against (Section 6: the
 * projections omega of Eq. (1) replaced by trainable vectors; with M == NULL, dW is exactly
 * that gradient).  The logits depend on W through w_j^T (M x') only, so
 *   dW[h][j][:] = sum over the batch and over all query and key rows of dlogit_j (M x')^T.
 *   dW: [H, m, r], or [m, r] (summed over the heads as well) when w_shared != 0; float32,
 *       overwritten; may be NULL, as may every other gradient pointer.
 * Everything else as dark_attn_bwd, including the workspace size.
 */
dark_status dark_attn_bwd_dw(const dark_params* p, int causal, const void* Q, const void* K,
                             const void* V, const float* M, const float* W, const void* dOut,
                             float* dQ, float* dK, float* dV, float* dM, float* dW,
                             void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Causal forward and backward as a pair (training): the backward needs the fp16 operand
 * copies of (M, W), the key norms and the exclusive prefix states of the key/value pass,
 * all of which the causal forward has just computed.  dark_attn_causal_fwd_save() is
 * dark_attn_causal_fwd() that leaves them in `saved` (device memory, 256-byte aligned, at
 * least dark_saved_bytes(p) bytes, owned by the caller); dark_attn_bwd_saved() is the causal
 * dark_attn_bwd_dw() that reads them from there instead of recomputing them.  The caller
 * guarantees that `saved` was written by dark_attn_causal_fwd_save() with the same
 * parameters and the same K, V, M, W and has not been modified since; results are then bit
 * for bit those of dark_attn_bwd_dw().
 * dark_saved_bytes() is 0 for parameters without such a hand-over (anything the fused
 * MFMA backward does not take: the two calls then behave exactly like
 * dark_attn_causal_fwd() and dark_attn_bwd_dw(causal = 1) and ignore `saved`, which may be
 * NULL).  Otherwise: DARK_EWORKSPACE if saved is NULL or too small, DARK_EALIGN if it is
 * misaligned.  The workspace sizes are those of the plain calls.
 */
size_t dark_saved_bytes(const dark_params* p);
dark_status dark_attn_causal_fwd_save(const dark_params* p, const void* Q, const void* K, const void* V,
                                      const float* M, const float* W, void* out,
                                      void* saved, size_t saved_bytes,
                                      void* ws, size_t ws_bytes, void* hip_stream);
dark_status dark_attn_bwd_saved(const dark_params* p, const void* Q, const void* K, const void* V,
                                const float* M, const float* W, const void* dOut,
                                const void* saved, size_t saved_bytes,
                                float* dQ, float* dK, float* dV, float* dM, float* dW,
                                void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Whitening geometry: an initial M from the statistics of the inputs (paper: Section 4.1
 * and Proposition C.1: with M the inverse square root of the input covariance Lambda, M q and
 * M k have identity covariance).  Per head h, over all B * L rows of Q and of K (pooled: the paper
 * assumes Cov(q) = Cov(k), Section 3; K may be NULL, then Q alone):
 *   Lambda_h = centred sample covariance (divisor = number of rows),
 *   Lambda_h = U diag(lambda) U^T with lambda descending, each lambda raised to at least
 *              1e-6 * lambda_1,
 *   M_h      = diag(lambda_1..r ^ -1/2) U[:, :r]^T      (so M Lambda M^T = I_r and, for r = d,
 *              M^T M = Lambda^-1; the rows of M are determined up to sign).
 * Uses p->B, H, L, d, r, io_dtype (Q, K: [B, H, L, d] in io_dtype); m, dv are ignored.
 *   M_out:   [H, r, d] float32.
 *   cov_out: [H, d, d] float32, receives Lambda; may be NULL.
 * Workspace: dark_workspace_bytes(p, DARK_OP_WHITEN, 0).  DARK_EUNSUPPORTED for d > 128 or
 * r > d; DARK_EINVAL for B * L == 0.  The estimator, the pooling and the floor are this
 * library's readings; the paper states only the population identity.
 */
dark_status dark_whiten(const dark_params* p, const void* Q, const void* K, float* M_out, float* cov_out,
                        void* ws, size_t ws_bytes, void* hip_stream);

/*
 * One token of causal attention as a recurrence (the causal form of the paper's linear
 * attention, Section 2, advanced by one position; serving).  Per (b, h), with the new query,
 * key and value of that position (q, k: [B, H, d], v: [B, H, dv], in io_dtype):
 *   S <- S + phi(k) v^T,   z <- z + phi(k),   out = phi(q)^T S / phi(q)^T z      (out: [B, H, dv], io_dtype)
 * which is row t of dark_attn_causal_fwd over the tokens seen so far.  The state belongs to the
 * caller: S [B, H, m, dv], z [B, H, m], c [B, H], all float32.  It is kept under one shift per
 * (b, h): S = sum_l exp(logit(k_l) - c) v_l^T with c (natural log) the largest key logit so far; start
 * with S = 0, z = 0, c = -infinity.  Keys more than ~87 nats below c vanish (fp32).  p->L is ignored;
 * p->out_dtype is ignored.  No workspace.  DARK_EUNSUPPORTED when 2 d + 2 r + 2 m + dv exceeds ~12000.
 * M may be NULL (identity, r == d).  fp32 arithmetic for every io_dtype.
 */
dark_status dark_decode_step(const dark_params* p, const void* q, const void* k, const void* v,
                             const float* M, const float* W, float* S, float* z, float* c,
                             void* out, void* hip_stream);

/*
 * Per-kernel device timing for benchmarks.  While enabled (on != 0) every kernel
 * launch of the library carries a start and a stop event that the launch itself
 * stamps with the kernel's begin and end on the device, and the launch stream is
 * synchronised before each such launch (so the entry points block the host and
 * the kernels no longer run back to back: enable it for measurement only).
 * dark_timing_read() synchronises with the recorded events, adds their elapsed
 * times into per-kernel totals and returns, for kernel slot `k`
 * (0 <= k < dark_timing_slots()), its name (static storage), the number of
 * launches and the summed milliseconds since the last dark_timing_reset().
 * Host pointers.  Not thread-safe; meant for single-threaded measurement only.
 */
void dark_timing_enable(int on);
void dark_timing_reset(void);
int dark_timing_slots(void);
dark_status dark_timing_read(int k, const char** name, int64_t* launches, double* total_ms);

/*
 * Measured ceilings of the device, for benchmarks that report the attention
 * kernels against what the chip sustains rather than against its data-sheet
 * peaks.  Plain kernels, no part of the attention path; each call enqueues one
 * launch on `hip_stream` and returns (time it with events on that stream).
 * Device pointers; nbytes a multiple of 16; `sink` is a device buffer of at
 * least 4 bytes that is (practically) never written.
 *   dark_ceiling_copy  reads nbytes from src and writes them to dst.
 *   dark_ceiling_read  reads nbytes from src.
 *   dark_ceiling_mfma  runs `iters` rounds of four independent 32x32x16 fp16
 *                      MFMAs in each of 2048 waves (eight per compute unit)
 *                      and stores the floating-point operations of the launch
 *                      in *flops (host pointer).
 * DARK_EINVAL for null pointers, nbytes not a multiple of 16 or iters < 0.
 */
dark_status dark_ceiling_copy(void* dst, const void* src, size_t nbytes, void* hip_stream);
dark_status dark_ceiling_read(const void* src, size_t nbytes, void* sink, void* hip_stream);
dark_status dark_ceiling_mfma(int iters, void* sink, double* flops, void* hip_stream);

/*
 * Wall-clock timeline of the two large kernels of the bidirectional MFMA forward,
 * for libraries built with -DDARK_TIMELINE (python -m paper_2603_04127_amd.timeline
 * builds one beside the ordinary library).  In such a build every wave of the
 * key/value pass (which = 0) and of the readout (which = 1) stores the device's
 * 100 MHz wall clock at fixed points of its run into a device array, 16 slots per
 * wave:
 *   which = 0: [workgroup (first 512)][wave (4)][slot]: 0 kernel start, 1 M' in LDS,
 *              2 first barrier passed, 3 tile loop begins, 4 tile loop done, 5 kernel end
 *   which = 1: [workgroup (first 256)][wave (8)][slot]: 0 kernel start, 1 first fill
 *              done, 2 + 3 i, 3 + 3 i, 4 + 3 i: unit loop begins, unit loop done, rows
 *              stored, for the wave's items i = 0, 1, 2; 15 kernel end
 * dark_timeline_read copies n slots (int64 ticks) of the last launch to `host`
 * (host pointer; synchronises the device).  The ordinary build records nothing
 * and returns DARK_EUNSUPPORTED.  DARK_EINVAL for a null pointer, an unknown
 * `which` or n beyond the array.
 */
dark_status dark_timeline_read(int which, int64_t* host, size_t n);

#ifdef __cplusplus
}
#endif
#endif /* DARK_H_ */

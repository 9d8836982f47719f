// Fused MFMA path of the DARK attention library (gfx950): bf16 inputs, fp32 accumulation.
//
// Per (b,h), with alpha = sqrt(scale), A = W M (Appendix B: omega~_j = M^T w_j) and
// everything kept in the log2 domain:
//   A' = alpha log2(e) A           (fp16 MFMA operand; x is bf16, exactly representable in fp16)
//   M' = alpha sqrt(log2(e)/2) M   so that n'(x) = |M' x|^2 = log2(e) * 1/2 |M x'|^2
//   key features    phi_K,lj = exp2(x_l . A'_j - n'(x_l) - c)      (Section 4.1 feature map)
//   query features  phi_Q,ij = exp2(x_i . A'_j + c - mu_i)
// c is a shift shared by a block of 64 features (chosen from the data, it cancels against the
// same shift on the query side) and mu_i a per-row shift (cancels in the ratio), so no
// exponential can overflow.  The query-side norm term is a per-row factor and is dropped.
//
// Kernels (Section 2, "Efficient attention via random feature kernels": K'^T V first, then Q'):
//   k_prep       A', M' for every head
//   k_kv_reduce  per (b,h, L-slice, 256-feature block): [S|z] += phi_K^T [V|1], features never
//                leave registers; MFMA 1 (projection) feeds MFMA 2 (phi^T V) through the
//                accumulator layout, which is already the operand layout after a bf16 pack
//   k_kv_merge   fixed-order merge of the slice states (deterministic), bf16 S^T for the readout
//   k_readout    per (b,h, token range): out = phi_Q S / phi_Q z
#include <cmath>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

// Wall-clock stamps for dark_timeline_read (builds with -DDARK_TIMELINE only).  Every lane stores the same value
// to the same slot, with no branch around the store: behind a lane test, or with the slot kept in a register
// across the loop, the compiler's register allocation of these kernels falls apart.
constexpr int kTlKvWgs = 512, kTlRoWgs = 256, kTlSlots = 16;
#ifdef DARK_TIMELINE
__device__ long long g_tl_kv[kTlKvWgs * 4 * kTlSlots];
__device__ long long g_tl_ro[kTlRoWgs * 8 * kTlSlots];
#define DARK_STAMP(arr, nwg, nwv, slot)                                                                          \
  __builtin_nontemporal_store((long long)wall_clock64(),                                                        \
                              arr + ((size_t)(blockIdx.x % (nwg)) * (nwv) + threadIdx.x / 64) * kTlSlots + (slot))
#else
#define DARK_STAMP(arr, nwg, nwv, slot) \
  do {                                   \
  } while (0)
#endif
#define KV_STAMP(slot) DARK_STAMP(g_tl_kv, kTlKvWgs, 4, slot)
#define RO_STAMP(slot) DARK_STAMP(g_tl_ro, kTlRoWgs, 8, slot)

// ---------------------------------------------------------------------------
// k_prep: A'[h][j][:] = alpha log2e sum_t W[h][j][t] M[h][t][:]  (fp16),  M' = alpha sqrt(log2e/2) M.
// One block per (h, 256 / (d/4) feature rows).  Every global load of the block (its W rows and all
// of M, as float4) is issued before the first wait, so the block pays the memory latency once;
// then thread (row, column group) accumulates four adjacent outputs over t from LDS.
// Requires r, d multiples of 4, d <= 256.
// ---------------------------------------------------------------------------
constexpr int kPrepMaxLoads = 16;  // float4 loads of M per thread: r * d / 4 / 256 <= 16 for r, d <= 128
__global__ __launch_bounds__(256) void k_prep(const float* __restrict__ M, const float* __restrict__ W,
                                              _Float16* __restrict__ Ah, _Float16* __restrict__ Mh, int m, int r,
                                              int d, int w_shared, float alpha) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int cg = d / 4, rows = 256 / cg;          // column groups of 4; feature rows per block
  float* Ws = reinterpret_cast<float*>(smem);     // [rows][r + 4]
  float* Mt = Ws + rows * (r + 4);                // [r][d]
  const int h = blockIdx.y;
  const int j0 = blockIdx.x * rows;
  const f32x4* Mp = reinterpret_cast<const f32x4*>(M + (size_t)h * r * d);
  const float* w = W + (w_shared ? 0 : (size_t)h * m * r);
  const int tid = threadIdx.x;
  const int nM = r * d / 4, nW = rows * r / 4;    // float4 counts
  f32x4 mv[kPrepMaxLoads], wv[2];
#pragma unroll
  for (int u = 0; u < kPrepMaxLoads; ++u) {
    const int i = tid + 256 * u;
    mv[u] = i < nM ? Mp[i] : f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = tid + 256 * u, jj = i / (r / 4), t4 = i % (r / 4);
    wv[u] = (i < nW && j0 + jj < m) ? *reinterpret_cast<const f32x4*>(w + (size_t)(j0 + jj) * r + 4 * t4)
                                    : f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int u = 0; u < kPrepMaxLoads; ++u) {
    const int i = tid + 256 * u;
    if (i < nM) *reinterpret_cast<f32x4*>(Mt + 4 * i) = mv[u];
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = tid + 256 * u, jj = i / (r / 4), t4 = i % (r / 4);
    if (i < nW) *reinterpret_cast<f32x4*>(Ws + jj * (r + 4) + 4 * t4) = wv[u];
  }
  if (blockIdx.x == 0) {
    const float f = alpha * sqrtf(0.5f * kLog2e);
#pragma unroll
    for (int u = 0; u < kPrepMaxLoads; ++u) {
      const int i = tid + 256 * u;
      if (i < nM) {
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        h4 o = {(_Float16)(mv[u][0] * f), (_Float16)(mv[u][1] * f), (_Float16)(mv[u][2] * f), (_Float16)(mv[u][3] * f)};
        *reinterpret_cast<h4*>(Mh + (size_t)h * r * d + 4 * i) = o;
      }
    }
  }
  __syncthreads();
  const int jj = tid / cg, cq = tid % cg;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
  for (int t = 0; t < r; ++t) {
    const float wt = Ws[jj * (r + 4) + t];
    const f32x4 mt = *reinterpret_cast<const f32x4*>(Mt + t * d + 4 * cq);
#pragma unroll
    for (int x = 0; x < 4; ++x) acc[x] = fmaf(wt, mt[x], acc[x]);
  }
  if (jj < rows && j0 + jj < m) {
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const float f = alpha * kLog2e;
    h4 o = {(_Float16)(acc[0] * f), (_Float16)(acc[1] * f), (_Float16)(acc[2] * f), (_Float16)(acc[3] * f)};
    *reinterpret_cast<h4*>(Ah + ((size_t)h * m + j0 + jj) * d + 4 * cq) = o;
  }
}

// ---------------------------------------------------------------------------
// k_kv_reduce  (d = r = dv = 64): [S|z] of one L-slice of one (b,h), software-pipelined.
// Workgroup = 4 waves x 64 features (wave w owns features [64w, 64w+64) of a 256-feature block); two
// workgroups per CU.  Features never leave registers: the projection's accumulators, packed to bf16,
// are an operand of the second MFMA.
//
// The unit of work is a block: 32 tokens x 32 features of one wave.  For block b
//   A(b)  projection  U = [x | n'_hi n'_lo 1 1] . [A'_j | -1 -1 -c_hi -c_lo]   (5 MFMA 32x32x16 f16:
//         the norm term of the token and the shift of the feature enter through eight extra
//         contraction slots, each as an fp16 pair hi + lo, so the accumulators start from the
//         constant zero and no vector instruction touches the logits before the exponential)
//   B(b)  max check, exp2, pack to bf16                                         (vector ALU)
//   C(b)  S += phi^T V (4 MFMA 32x32x16 bf16);  z is summed by the vector ALU beside the exponentials
// and iteration b issues C(b-1) and A(b+1) between the pieces of B(b), pinned by sched_barrier, so
// the matrix pipe and the vector ALU always have independent work from the same wave.
//
// Staging: thread (wave w, l16, g16) owns the 16-byte pieces g16 and 4 + g16 of key row 16 w + l16 of
// a tile: it loads them a tile ahead, converts bf16 -> fp16, stores them to LDS and, from the same
// registers, feeds the 16x16x32 MFMAs that give x~ = M' x of its wave's 16 rows; n' = |x~|^2 goes to
// the row's extra slots.  V tiles go global -> LDS directly (XOR-swizzled on the source side for the
// transposing reads).  One barrier per 64-token tile; X tiles are triple-buffered (tile t+1 is read
// by the last block of tile t, tile t+2 is being written), V tiles too (the last block of tile t-1
// still reads V(t-1) after the barrier).
// ---------------------------------------------------------------------------
struct KvSmem {
  static constexpr int XS = 88;  // fp16 per staged key row: 64 coordinates, 8 extra slots, 8 zeros, pad (conflict-free 16-byte reads)
  static constexpr int MS = 72;
  static constexpr size_t x_buf = (size_t)kTile * XS * 2;
  static constexpr size_t v_buf = (size_t)kTile * 64 * 2;
  static constexpr size_t x_bytes = 4 * x_buf;
  static constexpr size_t v_bytes = 3 * v_buf;
  static constexpr size_t m_bytes = (size_t)64 * MS * 2;
  static constexpr size_t total = x_bytes + v_bytes + m_bytes;
};
constexpr float kF16Max = 65504.f;
// The key pass looks at a feature's running sum z after every block instead of at the block's logits before the
// exponentials: below 2^64 (a single feature value above it, or 2^20 positions at 2^44, would cross it) the state
// is far from the end of the fp32 range even after the products with V; beyond it the feature's shift is raised
// by the block's largest logit, at least by 2^32.
constexpr float kZBig = 1.8446744073709552e19f;  // 2^64
constexpr float kZDown = 32.0f;

// TP: the partial state is written feature-contiguous ([bh][p][dv][m], the layout of the merged S^T) for
// k_kv_merge_t; otherwise [bh][p][m][dv], which the causal prefix kernel reads.
template <bool TP>
__global__ __launch_bounds__(256, 2) void k_kv_reduce(const unsigned short* __restrict__ Kg,
                                                    const unsigned short* __restrict__ Vg,
                                                    const _Float16* __restrict__ Ah, const _Float16* __restrict__ Mh,
                                                    unsigned short* __restrict__ Spart, float* __restrict__ zpart,
                                                    float* __restrict__ cpart, float* __restrict__ nrm_out, int H,
                                                    int L, int m, int P, int slice_len, int n_work, int n_first) {
  using SM = KvSmem;
  constexpr int D = 64, DV = 64, R = 64;
  constexpr int XROW = SM::XS * 2;  // bytes per staged key row
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* Xs = smem;
  unsigned char* Vt = smem + SM::x_bytes;
  _Float16* Ms = reinterpret_cast<_Float16*>(smem + SM::x_bytes + SM::v_bytes);

  KV_STAMP(0);
  const int nfb = m / 256;
  const int q8 = blockIdx.x / (8 * nfb), rem = blockIdx.x % (8 * nfb);
  const int fb = rem / 8, work = q8 * 8 + rem % 8;
  if (work >= n_work) return;
  const int bh = work / P, p = work % P;
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  const int ntile = (tok_end - tok_begin + kTile - 1) / kTile;

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int l16 = lane % 16, g16 = lane / 16;
  const int f0 = fb * 256 + wv * 64;

  // M' -> registers now, -> LDS in the prologue (after the tile fetches have been issued)
  u32x4 mreg[R * D / 8 / 256];
#pragma unroll
  for (int u = 0; u < R * D / 8 / 256; ++u) {
    const int ci = tid + 256 * u, row = ci / (D / 8), kc = ci % (D / 8);
    mreg[u] = *reinterpret_cast<const u32x4*>(Mh + ((size_t)h * R + row) * D + 8 * kc);
  }
  // A' fragments: feature = f0 + 32 ft + l32, k = 16 s + 8 hf + [0,8); fragment 4 holds the extra slots
  half8 afr[2][5];
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
#pragma unroll
    for (int s = 0; s < 4; ++s)
      afr[ft][s] = *reinterpret_cast<const half8*>(Ah + ((size_t)h * m + f0 + 32 * ft + l32) * D + 16 * s + 8 * hf);
  // extra slots of the feature side: -1, -1 (times n'_hi, n'_lo of the token), -c_hi, -c_lo (times 1, 1);
  // only the lower half-wave's eight slots are used.  Returns the shift the pair really represents.
  auto fold_frag = [&](float cc, float& c_eff) {
    cc = fminf(fmaxf(cc, -kF16Max), kF16Max);
    const _Float16 hi = (_Float16)cc;
    const _Float16 lo = (_Float16)(cc - (float)hi);
    c_eff = (float)hi + (float)lo;
    half8 f = {(_Float16)-1.f, (_Float16)-1.f, -hi, -lo, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    if (hf) f = half8{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    return f;
  };
  float c[2] = {0.f, 0.f};
  {
    float ce;
    afr[0][4] = fold_frag(0.f, ce);
    afr[1][4] = afr[0][4];
  }

  const unsigned short* Kb = Kg + (size_t)bh * L * D;
  const unsigned short* Vb = Vg + (size_t)bh * L * DV;
  auto load_k = [&](u32x4(&kr)[2], int tile) {
    const int tok = min(tok_begin + tile * kTile + 16 * wv + l16, tok_end - 1);
    const unsigned short* src = Kb + (size_t)tok * D + 8 * g16;
    kr[0] = *reinterpret_cast<const u32x4*>(src);
    kr[1] = *reinterpret_cast<const u32x4*>(src + 32);
  };
  // V tile -> LDS: lane i of a wave fills position i % 8 of row r0 + i / 8 with the row's 16-byte piece
  // (i % 8) ^ v_swz(row).  Rows past the end of the slice repeat its last row (their features are zero).
  auto dma_v = [&](int tile, int vb) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = 16 * wv + 8 * u + lane / 8;
      const int tok = min(tok_begin + tile * kTile + row, tok_end - 1);
      dma16_to_lds(Vb + (size_t)tok * DV + 8 * ((lane % 8) ^ v_swz<128>(row)), Vt + vb * SM::v_buf + (16 * wv + 8 * u) * 128);
    }
  };
  // Convert the fetched key rows, store them, and write n' of this wave's 16 rows into their extra slots.
  // x~^T = M' X^T by 16x16x32 MFMAs with the tokens as columns (lane l16 = token, registers = rows of M'),
  // so the sum of squares runs over registers; the four lane groups are added by one fp32 MFMA against ones.
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  // (prologue only: tiles 0 and 1 together, so that their two dependent chains interleave)
  auto stage01 = [&](const u32x4(&kr0)[2], const u32x4(&kr1)[2]) {
    f32x4 acc[2][R / 16];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      half8 mf[R / 16];
#pragma unroll
      for (int rt = 0; rt < R / 16; ++rt)
        mf[rt] = *reinterpret_cast<const half8*>(Ms + (16 * rt + l16) * SM::MS + 32 * s + 8 * g16);
#pragma unroll
      for (int tl2 = 0; tl2 < 2; ++tl2) {
        u32x4 cv = bf16x8_to_f16x8(tl2 ? kr1[s] : kr0[s]);
        *reinterpret_cast<u32x4*>(Xs + tl2 * SM::x_buf + (16 * wv + l16) * XROW + (32 * s + 8 * g16) * 2) = cv;
#pragma unroll
        for (int rt = 0; rt < R / 16; ++rt)
          acc[tl2][rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(mf[rt], *reinterpret_cast<half8*>(&cv),
                                                                s == 0 ? zero4 : acc[tl2][rt], 0, 0, 0);
      }
    }
    f32x4 tot[2];
#pragma unroll
    for (int tl2 = 0; tl2 < 2; ++tl2) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int rt = 0; rt < R / 16; rt += 2)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          s0 = fmaf(acc[tl2][rt][v], acc[tl2][rt][v], s0);
          s1 = fmaf(acc[tl2][rt + 1][v], acc[tl2][rt + 1][v], s1);
        }
      // D[i][tok] = sum over the four lane groups of their partial sums: every lane ends with n' of token l16
      tot[tl2] = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, s0 + s1, zero4, 0, 0, 0);
    }
#pragma unroll
    for (int tl2 = 0; tl2 < 2; ++tl2) {
      // rows past the end get the largest norm fp16 holds: their features are exp2(-65504 ...) = 0;
      // all four lane groups hold the same n' and write the same 16 bytes
      // A norm beyond the fp16 range turns into +inf: the token's features are exp2(-inf) = 0, which is their
      // value to within fp32 next to any key of ordinary norm (and 0/0 = NaN in the output if every key is so).
      const int tokn = tok_begin + tl2 * kTile + 16 * wv + l16;
      const float n = (tokn >= tok_end) ? kF16Max : tot[tl2][0];
      if (nrm_out != nullptr && fb == 0 && g16 == 0 && tokn < tok_end) nrm_out[(size_t)bh * L + tokn] = n;
      const _Float16 hi = (_Float16)n;
      const _Float16 lo = (float)hi > kF16Max ? (_Float16)0.f : (_Float16)(n - (float)hi);
      fp16x2 hl;
      hl[0] = hi;
      hl[1] = lo;
      const u32x4 w = {*reinterpret_cast<unsigned*>(&hl), 0x3c003c00u, 0u, 0u};  // n'_hi, n'_lo, 1, 1, 0 x 4
      *reinterpret_cast<u32x4*>(Xs + tl2 * SM::x_buf + (16 * wv + l16) * XROW + 128) = w;
    }
  };

  // per-lane byte offsets of the operand fetches
  const unsigned xoff = l32 * XROW + 16 * hf;   // + 32 s: fragment s < 4 of a key row
  const unsigned xoff4 = l32 * XROW + 128 + 16 * hf;  // the extra slots (lower half-wave) / the zeros behind them (upper)
  const int jj = l32 % 16, tl = 4 * hf + jj / 4, kq = 2 * (l32 / 16) + (jj % 4) / 2;
  unsigned voff[2];
  voff[0] = tl * 128 + 16 * (kq ^ v_swz<128>(tl)) + 8 * (jj % 2);
  voff[1] = tl * 128 + 16 * ((kq + 4) ^ v_swz<128>(tl)) + 8 * (jj % 2);

  f32x16 S[2][2], U[2];
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) S[ft][ct] = zero16;
  float zl[2] = {0.f, 0.f};  // z of feature f0 + 32 ft + l32 over this half-wave's token rows
  u32x4 pk[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) pk[a][b] = u32x4{0u, 0u, 0u, 0u};
  half8 xa[5];

  auto fetch_xa = [&](const unsigned char* xrows) {
#pragma unroll
    for (int s = 0; s < 4; ++s) xa[s] = *reinterpret_cast<const half8*>(xrows + xoff + 32 * s);
    xa[4] = *reinterpret_cast<const half8*>(xrows + xoff4);
  };
  auto fetch_bv = [&](u32x4(&bv)[2], const unsigned char* vrows, int hh) {
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const unsigned char* vr = vrows + voff[ct] + hh * 16 * 128;
      u32x2 lo = lds_read_tr16(reinterpret_cast<const unsigned short*>(vr));
      u32x2 hi = lds_read_tr16(reinterpret_cast<const unsigned short*>(vr + 8 * 128));
      bv[ct] = u32x4{lo[0], lo[1], hi[0], hi[1]};
    }
  };

  // --- prologue: tiles 0 and 1 staged, tile 2 in flight, V(0) on its way, A(block 0) -------------
  u32x4 kreg[2];
  u32x4 cvh[2];  // converted rows of the tile whose norms are being computed (this thread's two 16-byte pieces)
  {
    u32x4 k1[2];
    load_k(kreg, 0);
    load_k(k1, 1);
    load_k(cvh, 2);
    dma_v(0, 0);
#pragma unroll
    for (int u = 0; u < R * D / 8 / 256; ++u) {
      const int ci = tid + 256 * u, row = ci / (D / 8), kc = ci % (D / 8);
      *reinterpret_cast<u32x4*>(Ms + row * SM::MS + 8 * kc) = mreg[u];
    }
    // 16 zero bytes behind each row's extra slots (never written again): the upper half-wave, whose feature-side
    // extra slots are zero, reads these instead of the row's norm, which may be infinite (inf x 0 = NaN)
    *reinterpret_cast<u32x4*>(Xs + (tid / kTile) * SM::x_buf + (tid % kTile) * XROW + 144) = u32x4{0u, 0u, 0u, 0u};
    KV_STAMP(1);
    __syncthreads();  // M' is read by every wave's norm MFMAs
    KV_STAMP(2);
    stage01(kreg, k1);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      cvh[s2] = bf16x8_to_f16x8(cvh[s2]);
      *reinterpret_cast<u32x4*>(Xs + 2 * SM::x_buf + (16 * wv + l16) * XROW + (32 * s2 + 8 * g16) * 2) = cvh[s2];
    }
    load_k(kreg, 3);
  }
  // The A' fragments must have arrived before the loop: otherwise the compiler's wait for them sits
  // inside the loop body, where (the counter being in-order) it would also wait for the loads in flight.
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
#pragma unroll
    for (int s = 0; s < 4; ++s) asm volatile("" ::"v"(afr[ft][s]));
  __builtin_amdgcn_s_waitcnt(0x0F72);  // vmcnt(2): everything but the two loads of tile 2
  __syncthreads();
  KV_STAMP(3);
  fetch_xa(Xs);
#pragma unroll
  for (int s = 0; s < 5; ++s)
    U[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[s], afr[0][s], s == 0 ? zero16 : U[0], 0, 0, 0);
  u32x4 bva[2];  // V fragments (first 16 token rows) of the block whose C runs next; the first C adds zeros
  fetch_bv(bva, Vt, 0);

  // Staging of the following tiles, cut into pieces that ride along the 32 pieces of a tile's four
  // blocks (slot = 8 k + i):  norms of tile t+2 (its rows were converted during the previous tile):
  //   slots 0,4,8,12: fetch the M' fragments of 16 rows;  3,7,11,15: their two MFMAs;  6,10,14,18: squares;
  //   19: sum over the lane groups;  22: n' -> extra slots of X(t+2);
  // slots 24..31: convert the rows of tile t+3 word by word, store them, fetch tile t+4.
  half8 mf[2];
  f32x4 nacc = zero4, ntot = zero4;
  float sq0 = 0.f, sq1 = 0.f;
  int b0 = 0, b1 = 1, b2 = 2, b3 = 3;   // X buffers of tiles t .. t+3
  int v0 = 0, v1 = 1, v2 = 2;           // V buffers of tiles t, t+1, t-1
  auto stg = [&](int slot, int t) {
    if (slot < 16 && slot % 4 == 0) {
      const int rt = slot / 4;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
        mf[s2] = *reinterpret_cast<const half8*>(Ms + (16 * rt + l16) * SM::MS + 32 * s2 + 8 * g16);
    }
    if (slot < 16 && slot % 4 == 3) {
      nacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(mf[0], *reinterpret_cast<half8*>(&cvh[0]), zero4, 0, 0, 0);
      nacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(mf[1], *reinterpret_cast<half8*>(&cvh[1]), nacc, 0, 0, 0);
    }
    if (slot >= 6 && slot <= 18 && slot % 4 == 2) {
#pragma unroll
      for (int v = 0; v < 4; v += 2) {
        sq0 = fmaf(nacc[v], nacc[v], sq0);
        sq1 = fmaf(nacc[v + 1], nacc[v + 1], sq1);
      }
    }
    if (slot == 19) {
      ntot = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, sq0 + sq1, zero4, 0, 0, 0);
      sq0 = sq1 = 0.f;
    }
    if (slot == 22) {  // all four lane groups hold the same n' and write the same 16 bytes: no branch
      const int tokn = tok_begin + (t + 2) * kTile + 16 * wv + l16;
      const float n = (tokn >= tok_end) ? kF16Max : ntot[0];
      if (nrm_out != nullptr && fb == 0 && g16 == 0 && tokn < tok_end) nrm_out[(size_t)bh * L + tokn] = n;
      const _Float16 hi = (_Float16)n;   // +inf beyond the fp16 range (see the first tiles above)
      const _Float16 lo = (float)hi > kF16Max ? (_Float16)0.f : (_Float16)(n - (float)hi);
      fp16x2 hl;
      hl[0] = hi;
      hl[1] = lo;
      const u32x4 w = {*reinterpret_cast<unsigned*>(&hl), 0x3c003c00u, 0u, 0u};
      *reinterpret_cast<u32x4*>(Xs + b2 * SM::x_buf + (16 * wv + l16) * XROW + 128) = w;
    }
    if (slot >= 24) {
      const int s2 = (slot - 24) / 4, q = (slot - 24) % 4;
      cvh[s2][q] = pack_f16_from_bf16pair(kreg[s2][q]);
      if (q == 3)
        *reinterpret_cast<u32x4*>(Xs + b3 * SM::x_buf + (16 * wv + l16) * XROW + (32 * s2 + 8 * g16) * 2) = cvh[s2];
      if (slot == 31) load_k(kreg, t + 4);
    }
  };
  // Two workgroups share a CU, and the instruction arbiter serves the older wave first: the workgroup that
  // arrived second (the grid is dealt out in order, n_first workgroups fill the first slot of every CU) would
  // run at 60 % of the first one's pace and then finish alone, on a half-empty CU.  It takes the higher
  // priority for the first 70 % of its tiles, after which the two end together.
  const bool second = (int)blockIdx.x >= n_first;
  const int prio_tiles = (7 * ntile + 5) / 10;
  if (second) __builtin_amdgcn_s_setprio(1);
  for (int t = 0; t < ntile; ++t) {
    if (second && t == prio_tiles) __builtin_amdgcn_s_setprio(0);
    // the buffer indices are rotated at the end of the body and kept in scalar registers;
    // bp: buffer of V(t-1); the very first block adds zero features times V(0)
    const int bp = (t == 0) ? 0 : v2;
    dma_v(t + 1, v1);  // V(t+1) -> LDS; the key side of the staging rides along the blocks (stg)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int ft = k % 2, pft = ft ^ 1, nft = ft ^ 1, cur = k & 1, nxt = cur ^ 1;
      const unsigned char* vprev = Vt + ((k == 0) ? bp : v0) * SM::v_buf + ((k == 0) ? 32 : 32 * ((k - 1) / 2)) * 128;
      u32x4 bvb[2];
      fetch_bv(bvb, vprev, 1);
      __builtin_amdgcn_sched_barrier(0);
      // First half of C(k-1).  The shifted logits of the block are not examined before the exponentials:
      // a feature's shift is set from its first block (below) and found too low afterwards, from the sum z.
      S[pft][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pk[nxt][0]),
                                                          *reinterpret_cast<bf16x8*>(&bva[0]), S[pft][0], 0, 0, 0);
      S[pft][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pk[nxt][0]),
                                                          *reinterpret_cast<bf16x8*>(&bva[1]), S[pft][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // Raise the shift of every feature whose largest logit in U[cur] asks for it (all of them when the shift is
      // being set for the first time), rescale what the feature has accumulated, and move U[cur] to the new shift.
      auto reshift = [&](bool set, float zold) {
        float mall = U[cur][0];
#pragma unroll
        for (int v = 1; v < 15; v += 2) mall = max3(mall, U[cur][v], U[cur][v + 1]);
        mall = fmaxf(mall, U[cur][15]);
        const float m0 = fmaxf(mall, __shfl_xor(mall, 32, 64));
        // a feature whose sum has left the range is brought down by at least 2^kZDown even if this block's own
        // logits are small (its earlier blocks were the large ones)
        const bool over = !(fabsf(zl[ft] + __shfl_xor(zl[ft], 32, 64)) < kZBig);
        const float delta = set ? m0 : (over ? fmaxf(m0, kZDown) : (m0 > kRaise ? m0 : 0.f));
        float ceff;
        afr[ft][4] = fold_frag(c[ft] + delta, ceff);
        const float deff = ceff - c[ft];
        c[ft] = ceff;
#pragma unroll
        for (int v = 0; v < 16; ++v) U[cur][v] -= deff;
        if (!set) {
          const float f = fast_exp2(-deff);
          zl[ft] = zold * f;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float fr = __shfl(f, 8 * (v / 4) + 4 * hf + (v % 4), 64);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) S[ft][ct][v] *= fr;
          }
        }
      };
      if (t == 0 && k < 2) reshift(true, 0.f);  // workgroup-uniform
      const float zprev = zl[ft];
      __builtin_amdgcn_sched_barrier(0);
      // B(k), second part, in eight pieces; piece i follows MFMA i of A(k+1) (i < 5) or of C(k-1)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i < 5) {
          U[nxt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[i], afr[nft][i], i == 0 ? zero16 : U[nxt], 0, 0, 0);
        } else if (i < 7) {
          S[pft][i - 5] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pk[nxt][1]),
                                                                  *reinterpret_cast<bf16x8*>(&bvb[i - 5]), S[pft][i - 5], 0, 0, 0);
        }
        const float ea = fast_exp2(U[cur][2 * i]), eb = fast_exp2(U[cur][2 * i + 1]);
        pk[cur][i / 4][i % 4] = pack_bf16(ea, eb);
        zl[ft] = (zl[ft] + ea) + eb;
        // operand fetches for the next iteration, behind the last MFMAs that read the old ones
        if (i == 5 && k == 0) fetch_xa(Xs + b0 * SM::x_buf + 32 * XROW);  // second half of this tile
        if (i == 5 && k == 2) fetch_xa(Xs + b1 * SM::x_buf);              // first half of the next tile
        if (i == 6) fetch_bv(bva, Vt + v0 * SM::v_buf + 32 * (k / 2) * 128, 0);  // V rows of this block
        stg(8 * k + i, t);
        __builtin_amdgcn_sched_barrier(0);
      }
      // keep this block's results on this side of the next block's branch (the compiler would otherwise
      // sink the last exponentials to their first use, behind it)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int q = 0; q < 4; ++q) asm volatile("" : "+v"(pk[cur][hh][q]));
      asm volatile("" : "+v"(zl[ft]));
      // Rare: a sum that is no longer below 2^kZBig (or not finite: an exponential overflowed) means the shift of
      // some feature is too low.  Nothing of this block has reached S yet (C(k) is issued with the next block) and
      // U[cur] is intact, so the block is simply redone under the raised shift.
      if (__any(!(fabsf(zl[ft]) < kZBig))) {
        reshift(false, zprev);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float ea = fast_exp2(U[cur][2 * i]), eb = fast_exp2(U[cur][2 * i + 1]);
          pk[cur][i / 4][i % 4] = pack_bf16(ea, eb);
          zl[ft] = (zl[ft] + ea) + eb;
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F72);  // vmcnt(2): V(t+1) has landed; the two key loads may still fly
    __syncthreads();
    {
      const int r0 = b0, r2 = v2;
      b0 = __builtin_amdgcn_readfirstlane(b1);
      b1 = __builtin_amdgcn_readfirstlane(b2);
      b2 = __builtin_amdgcn_readfirstlane(b3);
      b3 = __builtin_amdgcn_readfirstlane(r0);
      v2 = __builtin_amdgcn_readfirstlane(v0);
      v0 = __builtin_amdgcn_readfirstlane(v1);
      v1 = __builtin_amdgcn_readfirstlane(r2);
    }
  }
  KV_STAMP(4);
  // drain: C of the last block (second half of the last tile, feature tile 1)
  {
    const unsigned char* vlast = Vt + v2 * SM::v_buf + 32 * 128;  // after the last rotation v2 is the last tile's buffer
    u32x4 bvb[2];
    fetch_bv(bvb, vlast, 1);
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
      S[1][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pk[1][0]),
                                                         *reinterpret_cast<bf16x8*>(&bva[ct]), S[1][ct], 0, 0, 0);
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
      S[1][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pk[1][1]),
                                                         *reinterpret_cast<bf16x8*>(&bvb[ct]), S[1][ct], 0, 0, 0);
  }

  // --- epilogue: partial state of this slice (bf16 in memory: half the bytes on the way to the merge;
  // the merged state is rounded to bf16 for the readout's MFMA anyway).  Each wave turns its 64 x dv
  // block through LDS (the tile buffers are free now) so that the stores are 16-byte pieces of whole rows.
  const size_t pbase = (size_t)bh * P + p;
  wait_vmcnt0();   // the key loads issued for tiles past the end
  __syncthreads();  // every wave is done with the tile buffers
  if (!TP) {
    constexpr int ROWB = DV * 2 + 16;
    static_assert(4 * 64 * ROWB <= SM::x_bytes + SM::v_bytes, "stage does not fit the tile buffers");
    unsigned char* stg = smem + wv * 64 * ROWB;
#pragma unroll
    for (int ft = 0; ft < 2; ++ft)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 32 * ft + 8 * (v / 4) + 4 * hf + (v % 4);
          *reinterpret_cast<unsigned short*>(stg + row * ROWB + (32 * ct + l32) * 2) =
              (unsigned short)(pack_bf16(S[ft][ct][v], 0.f) & 0xffffu);
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    constexpr int CPR = DV / 8;
#pragma unroll
    for (int k = 0; k < 64 * CPR / 64; ++k) {
      const int i = lane + 64 * k, row = i / CPR, ch = i % CPR;
      const u32x4 w = *reinterpret_cast<const u32x4*>(stg + row * ROWB + 16 * ch);
      *reinterpret_cast<u32x4*>(Spart + (pbase * m + f0 + row) * DV + 8 * ch) = w;
    }
  } else {
    // transposed: row = value column, the 64 features of this wave along the row (the accumulators hold four
    // consecutive features of one value column per register group: the stage is written 8 bytes at a time)
    constexpr int ROWB = 64 * 2 + 16;
    static_assert(4 * DV * ROWB <= SM::x_bytes + SM::v_bytes, "stage does not fit the tile buffers");
    unsigned char* stg = smem + wv * DV * ROWB;
#pragma unroll
    for (int ft = 0; ft < 2; ++ft)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const u32x2 w = {pack_bf16(S[ft][ct][4 * g], S[ft][ct][4 * g + 1]),
                           pack_bf16(S[ft][ct][4 * g + 2], S[ft][ct][4 * g + 3])};
          *reinterpret_cast<u32x2*>(stg + (32 * ct + l32) * ROWB + (32 * ft + 8 * g + 4 * hf) * 2) = w;
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < DV * 8 / 64; ++k) {
      const int i = lane + 64 * k, row = i / 8, ch = i % 8;
      const u32x4 w = *reinterpret_cast<const u32x4*>(stg + row * ROWB + 16 * ch);
      *reinterpret_cast<u32x4*>(Spart + (pbase * DV + row) * m + f0 + 8 * ch) = w;
    }
  }
#pragma unroll
  for (int ft = 0; ft < 2; ++ft) {
    const float zs = zl[ft] + __shfl_xor(zl[ft], 32, 64);
    if (hf == 0) zpart[pbase * m + f0 + 32 * ft + l32] = zs;
  }
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
    if (hf == 0) cpart[pbase * m + f0 + 32 * ft + l32] = c[ft];
  KV_STAMP(5);
}

// ---------------------------------------------------------------------------
// k_kv_merge: per (b,h, 64-feature block): c* = max over the slices and all features of the (b,h)
// of the per-feature shifts (one scalar per (b,h): on the query side it is a per-row factor that
// cancels);  S_j = sum_p 2^(c_pj - c*) S_pj (p ascending, fixed order), same for z.
// Writes S^T as bf16 [BH][DV][m] (the readout's MFMA operand), z [BH][m], c* [BH][m/64].
// ---------------------------------------------------------------------------
template <int DV>
__global__ __launch_bounds__(256) void k_kv_merge(const unsigned short* __restrict__ Spart,
                                                  const float* __restrict__ zpart, const float* __restrict__ cpart,
                                                  unsigned short* __restrict__ St, float* __restrict__ zt,
                                                  float* __restrict__ cf, int m, int P) {
  constexpr int PP = DV == 64 ? 16 : 8;  // slices per pass (one memory round trip each): as many as the registers hold
  __shared__ float tile[64][DV + 1];
  __shared__ float fac[PP][64];
  __shared__ float red[4];
  const int nblk = m / 64;
  const int bh = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int tid = threadIdx.x;
  constexpr int NV = 64 * DV / 8 / 256;  // 16-byte pieces (8 bf16 of one feature row) per thread and slice
  float acc[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  float zacc = 0.f;
  float cs = -INFINITY;
  for (int p0 = 0; p0 < P; p0 += PP) {
    const int np = min(PP, P - p0);
    // the pass's loads of the partial states are issued first: they do not depend on the shifts,
    // so their latency overlaps the reduction that finds c*
    u32x4 v[PP][NV];
    float zv[PP];
#pragma unroll
    for (int u = 0; u < PP; ++u) {
      const int pu = min(u, np - 1);
      const unsigned short* sp = Spart + (((size_t)bh * P + p0 + pu) * m + 64 * blk) * DV;
#pragma unroll
      for (int i = 0; i < NV; ++i) v[u][i] = *reinterpret_cast<const u32x4*>(sp + 8 * (tid + 256 * i));
      zv[u] = tid < 64 ? zpart[((size_t)bh * P + p0 + pu) * m + 64 * blk + tid] : 0.f;
    }
    if (p0 == 0) {
      // largest shift of the (b,h): P m values (m a multiple of 64), sixteen 16-byte loads in flight per thread
      const f32x4* cp4 = reinterpret_cast<const f32x4*>(cpart + (size_t)bh * P * m);
      const int n4 = P * m / 4;
      for (int i0 = tid; i0 < n4; i0 += 256 * 16) {
        f32x4 cv[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) cv[u] = cp4[min(i0 + 256 * u, n4 - 1)];
#pragma unroll
        for (int u = 0; u < 16; ++u) cs = fmaxf(fmaxf(cs, fmaxf(cv[u][0], cv[u][1])), fmaxf(cv[u][2], cv[u][3]));
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) cs = fmaxf(cs, __shfl_xor(cs, o, 64));
      if (tid % 64 == 0) red[tid / 64] = cs;
      __syncthreads();
      cs = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    } else {
      __syncthreads();  // the previous pass is done with fac
    }
    for (int i = tid; i < np * 64; i += 256)
      fac[i / 64][i % 64] = fast_exp2(cpart[((size_t)bh * P + p0 + i / 64) * m + 64 * blk + i % 64] - cs);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PP; ++u) {  // p ascending: the order of summation is fixed
      if (u < np) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const float f = fac[u][8 * (tid + 256 * i) / DV];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const unsigned w = v[u][i][j];
            acc[i][2 * j] = fmaf(f, __uint_as_float(w << 16), acc[i][2 * j]);
            acc[i][2 * j + 1] = fmaf(f, __uint_as_float(w & 0xffff0000u), acc[i][2 * j + 1]);
          }
        }
        if (tid < 64) zacc = fmaf(fac[u][tid], zv[u], zacc);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int e = 8 * (tid + 256 * i);
#pragma unroll
    for (int j = 0; j < 8; ++j) tile[e / DV][e % DV + j] = acc[i][j];
  }
  __syncthreads();
  constexpr int PER = 64 * DV / 256;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    int idx = tid + 256 * i;
    int cc = idx / 64, f = idx % 64;
    St[((size_t)bh * DV + cc) * m + 64 * blk + f] = (unsigned short)(pack_bf16(tile[f][cc], 0.f) & 0xffffu);
  }
  if (tid < 64) zt[(size_t)bh * m + 64 * blk + tid] = zacc;
  if (tid == 0) cf[(size_t)bh * nblk + blk] = cs;
}

// ---------------------------------------------------------------------------
// k_kv_merge_t: the same merge for feature-contiguous partial states [bh][p][dv][m] (dv = 64), which are
// already laid out like S^T: no transpose, and every load of the block is in flight before the first
// wait (one memory round trip; the kernel is pure latency).  One block per (b,h, 64-feature block),
// P <= kMergeTMaxP slices.
// ---------------------------------------------------------------------------
constexpr int kMergeTMaxP = 8;
template <int P>  // the number of slices, so that no thread requests a slice twice
__global__ __launch_bounds__(256) void k_kv_merge_t(const unsigned short* __restrict__ Spart,
                                                    const float* __restrict__ zpart, const float* __restrict__ cpart,
                                                    unsigned short* __restrict__ St, float* __restrict__ zt,
                                                    float* __restrict__ cf, int m) {
  constexpr int DV = 64, PP = P;
  static_assert(P >= 1 && P <= kMergeTMaxP, "slice count");
  __shared__ float fac[PP][64];
  __shared__ float red[4];
  const int nblk = m / 64;
  const int bh = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int tid = threadIdx.x;
  const size_t sbase = (size_t)bh * P;
  // thread t: 16-byte pieces (value column t / 8 and 32 + t / 8, features 8 (t % 8) .. + 7 of the block)
  const int row = tid / 8, fch = tid % 8;
  u32x4 v[PP][2];
  float cmine[PP], zmine[PP];
#pragma unroll
  for (int u = 0; u < PP; ++u) {
    const int pu = min(u, P - 1);
#pragma unroll
    for (int k = 0; k < 2; ++k)
      v[u][k] = *reinterpret_cast<const u32x4*>(Spart + ((sbase + pu) * DV + row + 32 * k) * m + 64 * blk + 8 * fch);
    cmine[u] = cpart[(sbase + pu) * m + 64 * blk + (tid % 64)];
    zmine[u] = zpart[(sbase + pu) * m + 64 * blk + (tid % 64)];
  }
  // c* over every slice and feature of the (b,h)
  float cs = -INFINITY;
  {  // P m values, m a multiple of 64: 16-byte loads, all of a round in flight together
    const f32x4* cp4 = reinterpret_cast<const f32x4*>(cpart + sbase * m);
    const int n4 = P * m / 4;
    for (int i0 = tid; i0 < n4; i0 += 256 * 4) {
      f32x4 cv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) cv[u] = cp4[min(i0 + 256 * u, n4 - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u) cs = fmaxf(fmaxf(cs, fmaxf(cv[u][0], cv[u][1])), fmaxf(cv[u][2], cv[u][3]));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cs = fmaxf(cs, __shfl_xor(cs, o, 64));
  if (tid % 64 == 0) red[tid / 64] = cs;
  __syncthreads();
  cs = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float zacc = 0.f;
#pragma unroll
  for (int u = 0; u < PP; ++u) {
    const float f = fast_exp2(cmine[u] - cs);
    if (tid < 64) fac[u][tid] = f;
    if (u < P) zacc = fmaf(f, zmine[u], zacc);   // p ascending
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < PP; ++u) {  // p ascending: the order of summation is fixed
      if (u < P) {
        const f32x4 f0 = *reinterpret_cast<const f32x4*>(&fac[u][8 * fch]);
        const f32x4 f1 = *reinterpret_cast<const f32x4*>(&fac[u][8 * fch + 4]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const unsigned w = v[u][k][j];
          const float fa = j < 2 ? f0[2 * j] : f1[2 * j - 4], fb = j < 2 ? f0[2 * j + 1] : f1[2 * j - 3];
          acc[2 * j] = fmaf(fa, __uint_as_float(w << 16), acc[2 * j]);
          acc[2 * j + 1] = fmaf(fb, __uint_as_float(w & 0xffff0000u), acc[2 * j + 1]);
        }
      }
    }
    const u32x4 o = {pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3]), pack_bf16(acc[4], acc[5]),
                     pack_bf16(acc[6], acc[7])};
    *reinterpret_cast<u32x4*>(St + ((size_t)bh * DV + row + 32 * k) * m + 64 * blk + 8 * fch) = o;
  }
  if (tid < 64) zt[(size_t)bh * m + 64 * blk + tid] = zacc;
  if (tid == 0) cf[(size_t)bh * nblk + blk] = cs;
}

// ---------------------------------------------------------------------------
// k_readout
// Workgroup = 4 waves; each wave owns 64 tokens per step and sweeps all features in blocks of 64:
//   U^T[feat][tok] = A' X^T (MFMA f16; A' from LDS, X fragments in registers, converted bf16->fp16)
//   phi^T = exp2(U^T + c_blk - mu_tok), mu a lazily raised running row shift
//   out^T[c][tok] += S^T[c][feat] phi^T[feat][tok] (MFMA bf16; S^T from LDS),  den += phi . z
// No barrier in the main loop.  The accumulators hold out^T (lane = token); each wave turns its
// tile through a private LDS stage so that the global stores are whole 128-byte rows.
// ---------------------------------------------------------------------------
template <int D, int DV>
struct RoSmem {
  static constexpr int AS = D + 8;
  static constexpr int stage_row = 128 + 8;                   // bytes: 64 bf16 or 32 fp32, plus pad
  // the per-wave output stage (fp32 output only: bf16 rows leave from registers): 16 tokens per pass in the
  // eight-wave kernels, whose operands leave no room for more, else 32
  __host__ __device__ static constexpr int stage_rows(int nw) { return nw == 8 ? 16 : 32; }
  __host__ __device__ static constexpr size_t stage_bytes(int nw) { return (size_t)stage_rows(nw) * stage_row; }
  __host__ __device__ static constexpr size_t a_bytes(int m) { return (size_t)m * AS * 2; }
  __host__ __device__ static constexpr size_t s_bytes(int m) { return (size_t)DV * (m + 4) * 2; }
  __host__ __device__ static constexpr size_t misc_bytes(int m) { return (size_t)m * 4 + 16 * (size_t)((m / 64 + 3) / 4); }  // z, shifts
  // nbuf copies of A', S^T, z and the shifts (two where the LDS allows: the next head and (b,h) are then
  // resident before the workgroup's run of items reaches them; the output stage is halved to make room)
  __host__ __device__ static size_t total(int m, int nw, int nbuf) {
    return nbuf * (a_bytes(m) + s_bytes(m) + misc_bytes(m)) + nw * stage_bytes(nw);
  }
};
template <int D, int NFB, int NW>
constexpr int ro_nbuf() { return (D == 64 && NFB == 1 && NW == 8) ? 2 : 1; }

template <int D, int DV, int NFB, bool OUT_BF16, int NW>
__global__ __launch_bounds__(64 * NW, 1) void k_readout(const unsigned short* __restrict__ Qg,
                                                       const _Float16* __restrict__ Ah,
                                                       const unsigned short* __restrict__ St,
                                                       const float* __restrict__ zt, const float* __restrict__ cf,
                                                       void* __restrict__ outp, int Bsz, int H, int L,
                                                       int chunks_per_bh, int n_items, int items_per_wg) {
  using SM = RoSmem<D, DV>;
  constexpr int m = 256 * NFB;
  constexpr int NBUF = ro_nbuf<D, NFB, NW>();
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // LDS: NBUF copies of A', then NBUF copies of (S^T, z, shifts), then the per-wave output stages
  constexpr size_t kABytes = SM::a_bytes(m);
  constexpr size_t kSBase = NBUF * kABytes;
  constexpr size_t kBufBytes = SM::s_bytes(m) + SM::misc_bytes(m);
  constexpr int SR = SM::stage_rows(NW);
  const int SS = m + 4;
  constexpr int NT = 64 * NW;

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  unsigned char* stage = smem + kSBase + NBUF * kBufBytes + wv * SM::stage_bytes(NW);
  const int l32 = lane % 32, hf = lane / 32;

  // Work items are (head, batch entry, 64 NW-token chunk) triples, head slowest, so that neighbouring
  // items share first the (b,h) and then at least the head.  A workgroup takes a contiguous run of
  // them: A' is refilled only when the run crosses into the next head, and S^T, z of the next (b,h) are
  // already resident when a second buffer exists (the run of a workgroup rarely spans more than two).
  // Workgroups are dealt to the eight XCDs round-robin; neighbouring runs of items (which share S^T, z and
  // A') go to workgroups of one XCD, so that its L2 fetches each of them once.
  if (NW == 8) RO_STAMP(0);
  const int nwg = gridDim.x;
  const int wg = nwg % 8 == 0 ? (blockIdx.x % 8) * (nwg / 8) + blockIdx.x / 8 : blockIdx.x;
  const int item_begin = wg * items_per_wg;
  const int item_end = min(n_items, item_begin + items_per_wg);
  auto bh_of = [&](int vb) { return (vb % Bsz) * H + vb / Bsz; };
  const int vb0 = item_begin / chunks_per_bh;
  int cur_vb = -1, cur_h = -1;
  // X fragments (B operand of the projection): token = t0 + 32 tt + l32, k = 16 s + 8 hf + [0,8).
  // The raw bf16 rows of the next tile are fetched into these registers during the last slot of
  // the current one (their last use is the projection of the last unit), so the fetch latency
  // hides behind the rest of the tile.
  half8 xf[2][D / 16];
  bool have_x = false;
  auto fetch_x = [&](int fbh, int ft0) {
    const unsigned short* Qf = Qg + (size_t)fbh * L * D;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int tok = min(ft0 + 32 * tt + l32, L - 1);  // rows past the end repeat the last row; never stored
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        u32x4 raw = *reinterpret_cast<const u32x4*>(Qf + (size_t)tok * D + 16 * s + 8 * hf);
        xf[tt][s] = *reinterpret_cast<half8*>(&raw);
      }
    }
  };
  // LDS fill: A' of head h (h >= 0), S^T, z, shifts of (b,h) bhA into buffer bufA and, with two buffers, of
  // bhB into bufB (each when >= 0).  Every load is issued before the first store, so a fill costs one
  // memory round trip.
  auto fill = [&](int h, int abuf, int h2, int bhA, int bufA, int bhB, int bufB) {
    constexpr int NA = m * D / 8 / NT;   // 16-byte pieces of A' per thread
    constexpr int NS = DV * m / 4 / NT;  // 8-byte pieces of S^T per thread
    constexpr int NZ = (m + NT - 1) / NT;
    static_assert(m * D / 8 % NT == 0 && DV * m / 4 % NT == 0, "fill assumes whole pieces per thread");
    if constexpr (NA > 4 || NS > 8) {
      // large operands: in passes of a few pieces per thread (all of them in flight at once would spill)
      if (h >= 0) {
        for (int c0 = tid; c0 < m * D / 8; c0 += NT * 4) {
          u32x4 v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int ci = c0 + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
            v[u] = *reinterpret_cast<const u32x4*>(Ah + ((size_t)h * m + row) * D + 8 * kc);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int ci = c0 + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
            *reinterpret_cast<u32x4*>(reinterpret_cast<_Float16*>(smem) + row * SM::AS + 8 * kc) = v[u];
          }
        }
      }
      if (bhA >= 0) {
        unsigned char* base = smem + kSBase + bufA * kBufBytes;
        unsigned short* sl = reinterpret_cast<unsigned short*>(base);
        float* zq = reinterpret_cast<float*>(base + SM::s_bytes(m));
        for (int c0 = tid; c0 < DV * m / 4; c0 += NT * 8) {
          u32x2 v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int ci = c0 + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
            v[u] = *reinterpret_cast<const u32x2*>(St + ((size_t)bhA * DV + row) * m + 4 * fc);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int ci = c0 + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
            *reinterpret_cast<u32x2*>(sl + row * SS + 4 * fc) = v[u];
          }
        }
        for (int i = tid; i < m; i += NT) zq[i] = zt[(size_t)bhA * m + i];
        for (int i = tid; i < m / 64; i += NT) zq[m + i] = cf[(size_t)bhA * (m / 64) + i];
      }
      return;
    }
    // (two buffers) h: A' of that head into buffer abuf; h2: A' of that head into the other one
    u32x4 av[NBUF][NA];
    u32x2 sv[NBUF][NS];
    float zv[NBUF][NZ], cv[NBUF];
#pragma unroll
    for (int q = 0; q < NBUF; ++q) {
      const int hq = q ? h2 : h;
      if (hq >= 0) {
#pragma unroll
        for (int u = 0; u < NA; ++u) {
          const int ci = tid + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
          av[q][u] = *reinterpret_cast<const u32x4*>(Ah + ((size_t)hq * m + row) * D + 8 * kc);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < NBUF; ++q) {
      const int bhq = q ? bhB : bhA;
      if (bhq >= 0) {
#pragma unroll
        for (int u = 0; u < NS; ++u) {
          const int ci = tid + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
          sv[q][u] = *reinterpret_cast<const u32x2*>(St + ((size_t)bhq * DV + row) * m + 4 * fc);
        }
#pragma unroll
        for (int u = 0; u < NZ; ++u) zv[q][u] = (tid + NT * u < m) ? zt[(size_t)bhq * m + tid + NT * u] : 0.f;
        cv[q] = tid < m / 64 ? cf[(size_t)bhq * (m / 64) + tid] : 0.f;
      }
    }
#pragma unroll
    for (int q = 0; q < NBUF; ++q) {
      const int hq = q ? h2 : h;
      if (hq >= 0) {
        _Float16* al = reinterpret_cast<_Float16*>(smem + (q ? abuf ^ 1 : abuf) * kABytes);
#pragma unroll
        for (int u = 0; u < NA; ++u) {
          const int ci = tid + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
          *reinterpret_cast<u32x4*>(al + row * SM::AS + 8 * kc) = av[q][u];
        }
      }
    }
#pragma unroll
    for (int q = 0; q < NBUF; ++q) {
      const int bhq = q ? bhB : bhA;
      if (bhq >= 0) {
        unsigned char* base = smem + kSBase + (q ? bufB : bufA) * kBufBytes;
        unsigned short* sl = reinterpret_cast<unsigned short*>(base);
        float* zq = reinterpret_cast<float*>(base + SM::s_bytes(m));
#pragma unroll
        for (int u = 0; u < NS; ++u) {
          const int ci = tid + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
          *reinterpret_cast<u32x2*>(sl + row * SS + 4 * fc) = sv[q][u];
        }
#pragma unroll
        for (int u = 0; u < NZ; ++u)
          if (tid + NT * u < m) zq[tid + NT * u] = zv[q][u];
        if (tid < m / 64) zq[m + tid] = cv[q];
      }
    }
  };
  if (item_begin >= item_end) return;  // workgroup-uniform
  // The first tile's rows are requested before the first LDS fill, so that the two cold fetches overlap.
  {
    const int t00 = (item_begin % chunks_per_bh) * NT + 64 * wv;
    if constexpr (NBUF == 2) {
      fetch_x(bh_of(vb0), t00);  // rows past the end repeat the last row (a tile past the end is never used)
      have_x = t00 < L;
    } else if (t00 < L) {
      fetch_x(bh_of(vb0), t00);
      have_x = true;
    }
  }
  const _Float16* Asl = reinterpret_cast<const _Float16*>(smem);
  const unsigned short* Stl = reinterpret_cast<const unsigned short*>(smem + kSBase);
  const float* zl = reinterpret_cast<const float*>(smem + kSBase + SM::s_bytes(m));
  const float* cl = zl + m;
  const int h0 = vb0 / Bsz;
  if constexpr (NBUF == 2) {
    // First fill, outside the item loop and free of branches: every load of both buffers is in flight before the
    // first wait, one memory round trip.  (Inside the loop the compiler has to assume that loads of an earlier
    // refill may still be pending on the same registers and waits before each group.)  Buffer 1 takes what the
    // next (b,h) of the run needs; when the run has no second (b,h) it takes the first one's once more.
    const bool two = (item_end - 1) / chunks_per_bh > vb0;
    const int hn = two ? (vb0 + 1) / Bsz : h0;
    const int bh2[2] = {bh_of(vb0), bh_of(two ? vb0 + 1 : vb0)};
    const int hh2[2] = {h0, hn};
    constexpr int NA = m * D / 8 / NT, NS = DV * m / 4 / NT;
    static_assert(NT >= m, "one z per thread");
    u32x4 av[2][NA];
    u32x2 sv[2][NS];
    float zv[2], cv[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (q == 1 && !two) break;  // workgroup-uniform: a run inside one (b,h) needs no second buffer
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int ci = tid + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
        av[q][u] = *reinterpret_cast<const u32x4*>(Ah + ((size_t)hh2[q] * m + row) * D + 8 * kc);
      }
#pragma unroll
      for (int u = 0; u < NS; ++u) {
        const int ci = tid + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
        sv[q][u] = *reinterpret_cast<const u32x2*>(St + ((size_t)bh2[q] * DV + row) * m + 4 * fc);
      }
      zv[q] = zt[(size_t)bh2[q] * m + min(tid, m - 1)];
      cv[q] = cf[(size_t)bh2[q] * (m / 64) + min(tid, m / 64 - 1)];
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (q == 1 && !two) break;
      _Float16* al = reinterpret_cast<_Float16*>(smem + q * kABytes);
      unsigned char* base = smem + kSBase + q * kBufBytes;
      unsigned short* sl = reinterpret_cast<unsigned short*>(base);
      float* zq = reinterpret_cast<float*>(base + SM::s_bytes(m));
#pragma unroll
      for (int u = 0; u < NA; ++u) {
        const int ci = tid + NT * u, row = ci / (D / 8), kc = ci % (D / 8);
        *reinterpret_cast<u32x4*>(al + row * SM::AS + 8 * kc) = av[q][u];
      }
#pragma unroll
      for (int u = 0; u < NS; ++u) {
        const int ci = tid + NT * u, row = ci / (m / 4), fc = ci % (m / 4);
        *reinterpret_cast<u32x2*>(sl + row * SS + 4 * fc) = sv[q][u];
      }
      if (tid < m) zq[tid] = zv[q];
      if (tid < m / 64) zq[m + tid] = cv[q];
    }
    __syncthreads();
    RO_STAMP(1);
    cur_vb = vb0;
    cur_h = h0;
    // (the A' of a second head sits in buffer (hn - h0) % 2 = 1, where the loop looks for it)
  }
  // Two waves share a SIMD and the arbiter serves the older one (waves 0 .. NW/2 - 1) first; the younger
  // half of the workgroup takes the higher priority for the first two thirds of the run, so that both halves
  // finish together instead of the younger one working its last item alone.
  const int prio_items = (2 * (item_end - item_begin) + 1) / 3;
  for (int item = item_begin; item < item_end; ++item) {
    if (NW == 8 && wv >= NW / 2) {
      if (item - item_begin < prio_items) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
    }
    const int vb = item / chunks_per_bh, chunk = item % chunks_per_bh;
    const int bh = bh_of(vb);
    if (vb != cur_vb) {
      const int h = vb / Bsz, k = vb - vb0, ha = h - h0;
      if (cur_vb < 0) {  // first fill (single-buffered kernels; with two buffers it happened before the loop)
        fill(h, 0, -1, bh, 0, -1, 1);
        __syncthreads();
      } else {
        const bool came_with_first = NBUF == 2 && k == 1;
        const bool need_a = h != cur_h && !came_with_first;
        const bool need_s = !came_with_first;
        if (need_a || need_s) {
          __syncthreads();  // everyone is done reading what is overwritten (the buffers of two steps back)
          fill(need_a ? h : -1, ha % NBUF, -1, need_s ? bh : -1, k % NBUF, -1, 0);
          __syncthreads();
        }
      }
      cur_vb = vb;
      cur_h = h;
      if constexpr (NBUF == 2) {
        Asl = reinterpret_cast<const _Float16*>(smem + (ha % NBUF) * kABytes);
        const unsigned char* base = smem + kSBase + (k % NBUF) * kBufBytes;
        Stl = reinterpret_cast<const unsigned short*>(base);
        zl = reinterpret_cast<const float*>(base + SM::s_bytes(m));
        cl = zl + m;
      }
    }
    const int t0 = chunk * NT + 64 * wv;
    const int wg_end = L;
    if (t0 >= L) {  // wave-uniform
      have_x = false;
      continue;
    }
    // the tile fetched ahead: the next one, or this one again when there is none (never used then)
    const bool more = item + 1 < item_end;
    const int nitem = more ? item + 1 : item;
    const int nbh = bh_of(nitem / chunks_per_bh), nt0 = (nitem % chunks_per_bh) * NT + 64 * wv;
    if (!have_x) fetch_x(bh, t0);
    have_x = false;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        u32x4 cv = bf16x8_to_f16x8(*reinterpret_cast<u32x4*>(&xf[tt][s]));
        xf[tt][s] = *reinterpret_cast<half8*>(&cv);
      }
    constexpr int CT = DV / 32;
    f32x16 O[CT][2];
    float den[2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // ---- fast path -----------------------------------------------------------------------
    // Units of 32 features.  For unit g:  P(g) projection MFMAs -> U,  E(g) exp2/pack/denominator
    // (vector ALU) -> pk,  S(g) second MFMAs -> O.  Slot g of the schedule issues S(g-1), then
    // P(g+1), with the 16 pieces of E(g) spread between the MFMAs, so the matrix pipe and the
    // vector ALU work on different units at the same time.  The fast path applies no shift at all: the
    // features are 2^u with u the projection itself (the key shift c* and any per-token shift are per-row
    // factors of numerator and denominator alike), which is exact in bf16/fp32 as long as nothing leaves the
    // exponent range.  A token whose logits do is seen afterwards as a non-finite or out-of-range
    // denominator, and then the whole tile is redone by the careful path below with a running row shift.
    {
      constexpr int NS = 4 * CT;        // S MFMAs per unit
      constexpr int NP = 2 * (D / 16);  // P MFMAs per unit
      constexpr int STEPS = NS + NP, PER = STEPS / 16;
      static_assert(STEPS % 16 == 0, "schedule assumes 16 exp pieces per slot");
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) O[ct][tt] = zero16;
      den[0] = den[1] = 0.f;
#pragma unroll
      for (int fb = 0; fb < NFB; ++fb) {
        const _Float16* Ab = Asl + (size_t)(256 * fb + l32) * SM::AS + 8 * hf;
        const unsigned short* Sb = Stl + (size_t)l32 * SS + 256 * fb + 4 * hf;
        const float* zb = zl + 256 * fb + 4 * hf;
        f32x16 U[2][2];        // [unit parity][tt]
        u32x4 pk[2][2][2];     // [unit parity][tt][hh]
        half8 af[D / 16];      // A' fragments of the unit being projected
        u32x4 sf[2][CT];       // S^T fragments of the unit being accumulated
        f32x4 zf[2];           // z of the features of the current and the next pair of pieces
        // prologue: P(0)
#pragma unroll
        for (int s2 = 0; s2 < D / 16; ++s2) af[s2] = *reinterpret_cast<const half8*>(Ab + 16 * s2);
        zf[0] = *reinterpret_cast<const f32x4*>(zb);
#pragma unroll
        for (int s2 = 0; s2 < D / 16; ++s2)
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
            U[0][tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[s2], xf[tt][s2], s2 == 0 ? zero16 : U[0][tt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (NW == 8 && fb == 0) RO_STAMP(item == item_begin ? 2 : item == item_begin + 1 ? 5 : 8);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
          const int cur = g & 1, nxt = cur ^ 1;
          if (g == 7 && fb == NFB - 1) {
            fetch_x(nbh, nt0);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int i = 0; i < STEPS; ++i) {
            if (i < NS) {
              if (g >= 1) {  // S(g-1)
                const int hh = i / (2 * CT), ct = (i / 2) % CT, tt = i % 2;
                O[ct][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&sf[hh][ct]),
                                                                    *reinterpret_cast<bf16x8*>(&pk[nxt][tt][hh]),
                                                                    O[ct][tt], 0, 0, 0);
              }
              // A' fragments for P(g+1), one every other step
              if (g < 7 && i % 2 == 0 && i / 2 < D / 16)
                af[i / 2] = *reinterpret_cast<const half8*>(Ab + (size_t)32 * (g + 1) * SM::AS + 16 * (i / 2));
            } else {
              const int ip = i - NS;
              if (g < 7) {  // P(g+1)
                const int s2 = ip / 2, tt = ip % 2;
                U[nxt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[s2], xf[tt][s2], s2 == 0 ? zero16 : U[nxt][tt], 0, 0, 0);
              }
              // S^T fragments for S(g), one every other step
              if (ip % 2 == 0 && ip / 2 < 2 * CT) {
                const int hh = (ip / 2) / CT, ct = (ip / 2) % CT;
                const unsigned short* sr = Sb + (size_t)32 * ct * SS + 32 * g + 16 * hh;
                u32x2 lo = *reinterpret_cast<const u32x2*>(sr);
                u32x2 hi = *reinterpret_cast<const u32x2*>(sr + 8);
                sf[hh][ct] = u32x4{lo[0], lo[1], hi[0], hi[1]};
              }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (i % PER == PER - 1) {  // piece e of E(g): registers 8 hh + 2 q, + 1 of tile tt
              // order (hh, q, tt), tt fastest: four consecutive pieces share one f32x4 of z
              const int e = i / PER, tt = e % 2, hh = e / 8, q = (e / 2) % 4;
              const int k = e / 4;  // = 2 hh + q / 2: features 8 k + 4 hf + [0,4) of the unit
              if (e % 4 == 0) {     // fetch the next group's z (the next unit's first group at the end)
                const int kn = (k + 1) % 4, gn = g + (k + 1) / 4;
                zf[(k + 1) % 2] = *reinterpret_cast<const f32x4*>(zb + 32 * (gn % 8) + 8 * kn);
              }
              const float a = fast_exp2(U[cur][tt][8 * hh + 2 * q]);
              const float b = fast_exp2(U[cur][tt][8 * hh + 2 * q + 1]);
              pk[cur][tt][hh][q] = pack_bf16(a, b);
              // plain fmas: a dot2 instruction stalls behind the MFMAs in flight (measured: one
              // v_dot2c per MFMA costs as much as six ordinary vector instructions)
              den[tt] = fmaf(a, zf[k % 2][2 * (q % 2)], den[tt]);
              den[tt] = fmaf(b, zf[k % 2][2 * (q % 2) + 1], den[tt]);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        // drain: S(7)
#pragma unroll
        for (int i = 0; i < NS; ++i) {
          const int hh = i / (2 * CT), ct = (i / 2) % CT, tt = i % 2;
          O[ct][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&sf[hh][ct]),
                                                              *reinterpret_cast<bf16x8*>(&pk[1][tt][hh]), O[ct][tt], 0, 0, 0);
        }
      }
    }
    if (NW == 8) RO_STAMP(item == item_begin ? 3 : item == item_begin + 1 ? 6 : 9);
    have_x = more;
    const float dt0 = den[0] + xor32(den[0]), dt1 = den[1] + xor32(den[1]);
    const bool redo = __any(!(dt0 > kDenLo && dt0 < kDenHi) || !(dt1 > kDenLo && dt1 < kDenHi));

    // ---- careful path: running per-token shift, raised whenever a block exceeds it by 2^kTau ---
    if (redo) {
    // The fragments hold raw rows fetched during the last unit: those of the next tile (fetch this one
    // again), or, when this is the workgroup's last tile, this tile's own once more.  Either way they are
    // bf16 and have to be converted.
    if (have_x) fetch_x(bh, t0);
    have_x = false;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        u32x4 cv = bf16x8_to_f16x8(*reinterpret_cast<u32x4*>(&xf[tt][s]));
        xf[tt][s] = *reinterpret_cast<half8*>(&cv);
      }
#pragma unroll
    for (int ct = 0; ct < DV / 32; ++ct)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[ct][tt][v] = 0.f;
    den[0] = den[1] = 0.f;
    // Running per-token shift of the log2-features (lane = token column; both half-waves agree).
    // Set from the first feature block, afterwards only raised when exceeded by more than 2^kTau.
    float mu[2] = {0.f, 0.f};

    for (int blk = 0; blk < m / 64; ++blk) {
      const float cb = cl[blk];
      // U^T[ft][tt]: rows = features 64 blk + 32 ft + 8 g + 4 hf + e, column = token 32 tt + l32.
      // Accumulators start at c_blk - mu_token, so the MFMA chain delivers shifted log2-features.
      f32x16 U[2][2];
#pragma unroll
      for (int ft = 0; ft < 2; ++ft)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const float init = cb - mu[tt];
#pragma unroll
          for (int v = 0; v < 16; ++v) U[ft][tt][v] = init;
        }
#pragma unroll
      for (int s = 0; s < D / 16; ++s)
#pragma unroll
        for (int ft = 0; ft < 2; ++ft) {
          half8 a = *reinterpret_cast<const half8*>(Asl + (64 * blk + 32 * ft + l32) * SM::AS + 16 * s + 8 * hf);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
            U[ft][tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xf[tt][s], U[ft][tt], 0, 0, 0);
        }
      float bm[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        float m0 = -INFINITY;
#pragma unroll
        for (int ft = 0; ft < 2; ++ft)
#pragma unroll
          for (int v = 0; v < 16; v += 2) m0 = max3(m0, U[ft][tt][v], U[ft][tt][v + 1]);
        bm[tt] = fmaxf(m0, __shfl_xor(m0, 32, 64));
      }
      const bool first = (blk == 0);
      if (__any(first || bm[0] > kTau || bm[1] > kTau)) {  // rare after the first block
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const float delta = (first || bm[tt] > kTau) ? bm[tt] : 0.f;
          mu[tt] += delta;
#pragma unroll
          for (int ft = 0; ft < 2; ++ft)
#pragma unroll
            for (int v = 0; v < 16; ++v) U[ft][tt][v] -= delta;
          if (!first) {
            const float f = fast_exp2(-delta);
            den[tt] *= f;
#pragma unroll
            for (int ct = 0; ct < DV / 32; ++ct)
#pragma unroll
              for (int v = 0; v < 16; ++v) O[ct][tt][v] *= f;
          }
        }
      }
      // features, denominator, pack
      u32x4 pk[2][2][2];  // [ft][tt][hh]
#pragma unroll
      for (int ft = 0; ft < 2; ++ft)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 zv = *reinterpret_cast<const f32x4*>(zl + 64 * blk + 32 * ft + 8 * g + 4 * hf);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            float a0 = fast_exp2(U[ft][tt][4 * g + 0]);
            float a1 = fast_exp2(U[ft][tt][4 * g + 1]);
            float a2 = fast_exp2(U[ft][tt][4 * g + 2]);
            float a3 = fast_exp2(U[ft][tt][4 * g + 3]);
            const unsigned p0 = pack_bf16(a0, a1), p1 = pack_bf16(a2, a3);
            pk[ft][tt][g / 2][2 * (g % 2)] = p0;
            pk[ft][tt][g / 2][2 * (g % 2) + 1] = p1;
            den[tt] = fmaf(a3, zv[3], fmaf(a2, zv[2], fmaf(a1, zv[1], fmaf(a0, zv[0], den[tt]))));
          }
        }
      // out^T[ct][tt] += S^T phi^T : k-slot s of half hf is feature 64 blk + 32 ft + 16 hh + 8 (s/4) + 4 hf + s%4
#pragma unroll
      for (int ft = 0; ft < 2; ++ft)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
          for (int ct = 0; ct < DV / 32; ++ct) {
            const unsigned short* sr = Stl + (32 * ct + l32) * SS + 64 * blk + 32 * ft + 16 * hh + 4 * hf;
            u32x2 lo = *reinterpret_cast<const u32x2*>(sr);
            u32x2 hi = *reinterpret_cast<const u32x2*>(sr + 8);
            u32x4 av = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
              O[ct][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&av),
                                                                  *reinterpret_cast<bf16x8*>(&pk[ft][tt][hh]),
                                                                  O[ct][tt], 0, 0, 0);
          }
    }
    }  // careful path
    // normalise, turn through the wave's LDS stage, store whole rows.  Register v of O[ct][tt] is
    // out[token 32 tt + l32][c = 32 ct + 8 (v/4) + 4 hf + v%4].
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const float inv = 1.f / (den[tt] + xor32(den[tt]));
      const int row = lane / 8, ch = lane % 8;  // read side: 8 lanes per token row, 16 bytes each
      constexpr int NHP = 32 / SR;              // passes of SR tokens through the stage
#pragma unroll
      for (int hp = 0; hp < NHP; ++hp) {
        const bool mine = NHP == 1 || l32 / SR == hp;
        const int srow = l32 % SR;
        if (OUT_BF16) {
          // bf16 output: no LDS turn.  A lane holds, per block of 32 columns, four 8-byte pieces of its token's
          // row (columns 8 g + 4 hf + [0,4)); swapping halves between lanes l and l + 32 (v_permlane32_swap)
          // joins the two pieces of an even g in the lower lane and those of the odd g in the upper one, so
          // every lane stores 16 contiguous bytes and a store instruction covers 32-byte runs of 32 rows.
          if (hp == 0) {
            const int tok = t0 + 32 * tt + l32;
            unsigned short* orow = reinterpret_cast<unsigned short*>(outp) + ((size_t)bh * L + min(tok, L - 1)) * DV + 8 * hf;
#pragma unroll
            for (int ct = 0; ct < DV / 32; ++ct)
#pragma unroll
              for (int gp = 0; gp < 2; ++gp) {
                const int g0 = 2 * gp, g1 = g0 + 1;
                const unsigned a0 = pack_bf16(O[ct][tt][4 * g0] * inv, O[ct][tt][4 * g0 + 1] * inv);
                const unsigned a1 = pack_bf16(O[ct][tt][4 * g0 + 2] * inv, O[ct][tt][4 * g0 + 3] * inv);
                const unsigned b0 = pack_bf16(O[ct][tt][4 * g1] * inv, O[ct][tt][4 * g1 + 1] * inv);
                const unsigned b1 = pack_bf16(O[ct][tt][4 * g1 + 2] * inv, O[ct][tt][4 * g1 + 3] * inv);
                const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                const u32x4 w = {s0[0], s1[0], s0[1], s1[1]};
                // streaming store: the output is not read again by this launch, and lines left dirty in the
                // L2 would all be written back at the end of the kernel, on the critical path of the step
                if (tok < wg_end) *reinterpret_cast<u32x4*>(orow + 32 * ct + 16 * gp) = w;
              }
          }
        } else {
#pragma unroll
          for (int ct = 0; ct < DV / 32; ++ct) {
            if (mine) {
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                f32x4 w = {O[ct][tt][4 * g] * inv, O[ct][tt][4 * g + 1] * inv, O[ct][tt][4 * g + 2] * inv,
                           O[ct][tt][4 * g + 3] * inv};
                *reinterpret_cast<f32x4*>(stage + srow * SM::stage_row + (8 * g + 4 * hf) * 4) = w;
              }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < SR / 8; ++ps) {
              const int tok = t0 + 32 * tt + SR * hp + 8 * ps + row;
              f32x4 w = *reinterpret_cast<const f32x4*>(stage + (8 * ps + row) * SM::stage_row + 16 * ch);
              if (tok < wg_end)
                __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(reinterpret_cast<float*>(outp) +
                                                                        ((size_t)bh * L + tok) * DV + 32 * ct + 4 * ch));
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
          }
        }
      }
    }
    if (NW == 8) RO_STAMP(item == item_begin ? 4 : item == item_begin + 1 ? 7 : 10);
  }
  if (NW == 8) RO_STAMP(15);
}

constexpr size_t kLdsMax = 160 * 1024;
constexpr int kNumCU = 256;  // compute units of the MI355X

struct Plan {
  int P, slice_len, nfb, n_work, kv_grid;
  bool tp;  // partial states feature-contiguous, merged by k_kv_merge_t
  int ro_nw, chunks_per_bh, n_items, items_per_wg, ro_grid;
};

Plan make_plan(const Problem& pb) {
  const dark_params& p = pb.p;
  Plan pl{};
  pl.nfb = p.m / 256;
  const long long BH = pb.BH();
  // K pass: about two workgroups per CU (256 CUs); slices are whole tiles.
  // (d = 128: the 8-wave slice-state kernel, one workgroup per CU)
  int target = p.sched_kv_wgs > 0 ? p.sched_kv_wgs : (p.d == 128 ? 256 : 512);
  long long want = target / (BH * pl.nfb);  // rounding down keeps all workgroups co-resident
  if (want < 1) want = 1;
  int sl = (int)((p.L + want - 1) / want);
  sl = ((sl + kTile - 1) / kTile) * kTile;
  pl.slice_len = sl;
  pl.P = (p.L + sl - 1) / sl;
  pl.n_work = (int)(BH * pl.P);
  pl.kv_grid = ((pl.n_work + 7) / 8) * 8 * pl.nfb;
  pl.tp = p.d == 64 && pl.P <= kMergeTMaxP;
  // readout: (b,h, 256-token chunk) items dealt out in contiguous runs to about as many
  // workgroups as fit on the chip at once
  // one workgroup per CU: eight waves when the registers (d = 64) and the LDS allow, else four
  pl.ro_nw = p.d == 64 ? 8 : 4;
  const int ro_tok = 64 * pl.ro_nw;
  pl.chunks_per_bh = (p.L + ro_tok - 1) / ro_tok;
  pl.n_items = (int)(BH * pl.chunks_per_bh);
  const int ro_wgs = p.sched_ro_wgs > 0 ? p.sched_ro_wgs : 256;
  pl.items_per_wg = (pl.n_items + ro_wgs - 1) / ro_wgs;
  pl.ro_grid = (pl.n_items + pl.items_per_wg - 1) / pl.items_per_wg;
  return pl;
}

struct FusedBufs {
  _Float16* Ah;
  _Float16* Mh;
  unsigned short* Spart;  // per-slice partial states, bf16
  float* zpart;
  float* cpart;
  unsigned short* St;
  float* zt;
  float* cf;
  float* nrm;  // key norms [BH][L], d = 128 only
  float* nrm_out;  // where the key pass leaves the key norms it computes (causal callers), else null
};

void plan_bufs(const Problem& pb, const Plan& pl, Arena& ar, FusedBufs& b) {
  const dark_params& p = pb.p;
  const size_t BH = (size_t)pb.BH();
  b.Ah = ar.take<_Float16>((size_t)p.H * p.m * p.d);
  b.Mh = ar.take<_Float16>((size_t)p.H * p.r * p.d);
  b.Spart = ar.take<unsigned short>(BH * pl.P * p.m * p.dv);
  b.zpart = ar.take<float>(BH * pl.P * p.m);
  b.cpart = ar.take<float>(BH * pl.P * p.m);
  b.St = ar.take<unsigned short>(BH * p.dv * p.m);
  b.zt = ar.take<float>(BH * p.m);
  b.cf = ar.take<float>(BH * (p.m / 64));
  b.nrm = p.d == 128 ? ar.take<float>(BH * (size_t)(p.L > 0 ? p.L : 1)) : nullptr;
}

dark_status launch_kv(const Problem& pb, const Plan& pl, const FusedBufs& b, const void* K, const void* V) {
  const dark_params& p = pb.p;
  if (pl.tp) {
    DARK_TRY(allow_lds(k_kv_reduce<true>, KvSmem::total));
    DARK_LAUNCH(KID_KV_REDUCE, pb.st, k_kv_reduce<true>, dim3(pl.kv_grid), dim3(256), KvSmem::total,
                (const unsigned short*)K, (const unsigned short*)V, b.Ah, b.Mh, b.Spart, b.zpart, b.cpart, b.nrm_out, p.H,
                p.L, p.m, pl.P, pl.slice_len, pl.n_work, kNumCU);
  } else {
    DARK_TRY(allow_lds(k_kv_reduce<false>, KvSmem::total));
    DARK_LAUNCH(KID_KV_REDUCE, pb.st, k_kv_reduce<false>, dim3(pl.kv_grid), dim3(256), KvSmem::total,
                (const unsigned short*)K, (const unsigned short*)V, b.Ah, b.Mh, b.Spart, b.zpart, b.cpart, b.nrm_out, p.H,
                p.L, p.m, pl.P, pl.slice_len, pl.n_work, kNumCU);
  }
  return DARK_OK;
}

template <int D, int DV, int NFB, int NW>
dark_status launch_ro(const Problem& pb, const Plan& pl, const FusedBufs& b, const void* Q, void* out) {
  const dark_params& p = pb.p;
  const size_t lds = RoSmem<D, DV>::total(p.m, NW, ro_nbuf<D, NFB, NW>());
  const unsigned grid = (unsigned)pl.ro_grid;
  if (p.out_dtype == DARK_BF16) {
    auto kern = k_readout<D, DV, NFB, true, NW>;
    DARK_TRY(allow_lds(kern, lds));
    DARK_LAUNCH(KID_READOUT, pb.st, kern, dim3(grid), dim3(64 * NW), lds, (const unsigned short*)Q, b.Ah, b.St, b.zt,
                b.cf, out, p.B, p.H, p.L, pl.chunks_per_bh, pl.n_items, pl.items_per_wg);
  } else {
    auto kern = k_readout<D, DV, NFB, false, NW>;
    DARK_TRY(allow_lds(kern, lds));
    DARK_LAUNCH(KID_READOUT, pb.st, kern, dim3(grid), dim3(64 * NW), lds, (const unsigned short*)Q, b.Ah, b.St, b.zt,
                b.cf, out, p.B, p.H, p.L, pl.chunks_per_bh, pl.n_items, pl.items_per_wg);
  }
  return DARK_OK;
}

}  // namespace

dark_status fused_launch_prep(const Problem& pb, const float* M, const float* W, _Float16* Ah, _Float16* Mh) {
  const dark_params& p = pb.p;
  const int prep_rows = 256 / (p.d / 4);
  const int nA = (p.m + prep_rows - 1) / prep_rows;
  const size_t prep_lds = ((size_t)prep_rows * (p.r + 4) + (size_t)p.r * p.d) * sizeof(float);
  DARK_TRY(allow_lds(k_prep, prep_lds));
  DARK_LAUNCH(KID_PREP, pb.st, k_prep, dim3(nA, p.H), dim3(256), prep_lds, M, W, Ah, Mh, p.m, p.r, p.d, p.w_shared,
              std::sqrt(pb.scale));
  return DARK_OK;
}

bool fused_supported(const Problem& pb, int op, bool causal) {
  const dark_params& p = pb.p;
  if (op == DARK_OP_ATTN_CAUSAL_FWD) return fused_causal_supported(pb);
  if (op != DARK_OP_ATTN_FWD || causal) return false;
  if (p.io_dtype != DARK_BF16) return false;
  const bool shape64 = p.d == 64 && p.r == 64 && p.dv == 64;
  const bool shape128 = p.d == 128 && p.r == 128 && p.dv == 128;
  if (!shape64 && !shape128) return false;
  // feature counts the readout is instantiated for (its operands must fit the 160 KB of LDS)
  if (!(p.m == 256 || (shape64 && p.m == 512))) return false;
  return true;
}

dark_status fused_attn_fwd(const Problem& pb, Arena& ar, const void* Q, const void* K, const void* V,
                           const float* M, const float* W, void* out) {
  const dark_params& p = pb.p;
  const Plan pl = make_plan(pb);
  FusedBufs b{};
  plan_bufs(pb, pl, ar, b);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;

  DARK_TRY(fused_launch_prep(pb, M, W, b.Ah, b.Mh));
  if (p.d == 64) {
    DARK_TRY(launch_kv(pb, pl, b, K, V));
  } else {
    DARK_TRY(fused_launch_slice_state128(pb, K, V, b.Ah, b.Mh, b.nrm, b.Spart, b.zpart, b.cpart, pl.P, pl.slice_len));
  }
  const unsigned mgrid = (unsigned)(pb.BH() * (p.m / 64));
  if (pl.tp) {
#define DARK_MERGE_T(PV)                                                                                              \
  case PV:                                                                                                           \
    DARK_LAUNCH(KID_KV_MERGE, pb.st, k_kv_merge_t<PV>, dim3(mgrid), dim3(256), 0, b.Spart, b.zpart, b.cpart, b.St, \
                b.zt, b.cf, p.m);                                                                                    \
    break;
    switch (pl.P) {
      DARK_MERGE_T(1) DARK_MERGE_T(2) DARK_MERGE_T(3) DARK_MERGE_T(4) DARK_MERGE_T(5) DARK_MERGE_T(6) DARK_MERGE_T(7)
      DARK_MERGE_T(8)
      default: return DARK_EUNSUPPORTED;
    }
#undef DARK_MERGE_T
  } else if (p.dv == 64)
    DARK_LAUNCH(KID_KV_MERGE, pb.st, k_kv_merge<64>, dim3(mgrid), dim3(256), 0, b.Spart, b.zpart, b.cpart, b.St,
                b.zt, b.cf, p.m, pl.P);
  else
    DARK_LAUNCH(KID_KV_MERGE, pb.st, k_kv_merge<128>, dim3(mgrid), dim3(256), 0, b.Spart, b.zpart, b.cpart, b.St,
                b.zt, b.cf, p.m, pl.P);
  if (p.d == 64 && p.m == 256) {
    DARK_TRY((launch_ro<64, 64, 1, 8>(pb, pl, b, Q, out)));
  } else if (p.d == 64) {
    DARK_TRY((launch_ro<64, 64, 2, 8>(pb, pl, b, Q, out)));
  } else {
    DARK_TRY((launch_ro<128, 128, 1, 4>(pb, pl, b, Q, out)));
  }
  return DARK_OK;
}

dark_status fused_launch_kv_reduce(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                   const _Float16* Mh, unsigned short* Spart, float* zpart, float* cpart, int P,
                                   int slice_len, float* nrm_out) {
  const dark_params& p = pb.p;
  Plan pl{};
  pl.nfb = p.m / 256;
  pl.P = P;
  pl.slice_len = slice_len;
  pl.n_work = (int)(pb.BH() * P);
  pl.kv_grid = ((pl.n_work + 7) / 8) * 8 * pl.nfb;
  pl.tp = false;
  FusedBufs b{};
  b.Ah = const_cast<_Float16*>(Ah);
  b.Mh = const_cast<_Float16*>(Mh);
  b.Spart = Spart;
  b.zpart = zpart;
  b.cpart = cpart;
  b.nrm_out = nrm_out;
  if (p.d != 64) return DARK_EUNSUPPORTED;
  return launch_kv(pb, pl, b, K, V);
}

}  // namespace dark

extern "C" dark_status dark_timeline_read(int which, int64_t* host, size_t n) {
  using namespace dark;
  if (host == nullptr || (which != 0 && which != 1)) return DARK_EINVAL;
  const size_t cap = which == 0 ? (size_t)kTlKvWgs * 4 * kTlSlots : (size_t)kTlRoWgs * 8 * kTlSlots;
  if (n > cap) return DARK_EINVAL;
#ifdef DARK_TIMELINE
  static_assert(sizeof(long long) == sizeof(int64_t), "tick type");
  const hipError_t e = which == 0 ? hipMemcpyFromSymbol(host, HIP_SYMBOL(g_tl_kv), n * sizeof(int64_t), 0, hipMemcpyDeviceToHost)
                                  : hipMemcpyFromSymbol(host, HIP_SYMBOL(g_tl_ro), n * sizeof(int64_t), 0, hipMemcpyDeviceToHost);
  return e == hipSuccess ? DARK_OK : DARK_EHIP;
#else
  return DARK_EUNSUPPORTED;
#endif
}

// Fused MFMA backward of the causal DARK attention (gfx950): bf16 inputs, fp32 accumulation, fp32 gradients.
// d = r = dv = 64, m = 256.  No [rows, m] matrix is ever written to memory: features, their gradients and
// the 32 x 32 tiles of kernel values live in LDS and registers of the workgroup that walks a slice.
//
// Notation (per (b,h); the paper makes M learnable, Section 4, and fixes the feature map in Section 4.1;
// the gradients are the chain rule through that definition and the causal prefix form of Section 2's
// factorisation).  With a_il = phi(q_i).phi(k_l) for l <= i, D_i = sum_l a_il, out_i = sum_l a_il v_l / D_i
// and G = dOut:
//   da_il = (G_i.v_l + gd_i) / D_i,  gd_i = -G_i.out_i
//   phihat_Q,i = phi_Q,i / D_i                      (so phihat_Q,i . phi_K,l = a_il / D_i)
//   dlogit_Q,ij = phihat_Q,ij [ (S_<=i G_i)_j + gd_i z_<=i,j ],   S_<=i = sum_{l<=i} phi_K,l v_l^T, z likewise
//   dlogit_K,lj = phi_K,lj   [ (Rn_>=l v_l)_j + Rd_>=l,j ],       Rn_>=l = sum_{i>=l} phihat_Q,i G_i^T,
//                                                                 Rd_>=l = sum_{i>=l} phihat_Q,i gd_i
//   dV_l = Rn_>=l^T phi_K,l
//   dQ_i = alpha A^T dlogit_Q,i;   dK_l = alpha A^T dlogit_K,l - s_l alpha^2 M^T M k_l,  s_l = sum_j dlogit_K,lj
//   dM   = alpha W^T T - alpha^2 M Rm,  T = sum_tokens dlogit x^T (queries and keys),  Rm = sum_l s_l k_l k_l^T
// (the derivative through a query's norm term vanishes identically: scaling all features of a query leaves
// out_i unchanged).  Sums over l <= i split into the keys before the tile (running state, forward order) and
// the keys of the tile (masked 32 x 32 blocks); sums over i >= l likewise in reverse order.
//
// Kernels, after the key norms, the slice states and their exclusive prefix of the causal forward path:
//   k_bwd_fwd     per (b,h, slice), tiles in forward order: D_i, out_i, dQ, the query half of T, the slice's
//                 contribution to Rn, Rd; leaves lambda_i = log2 of the denominator (with the row shift) and
//                 gd_i per token for the reverse pass
//   k_bwd_suffix  exclusive suffix sums of the slices' Rn, Rd contributions
//   k_bwd_rev     per (b,h, slice), tiles in reverse order: dV, dK, the key half of T, Rm
//   k_bwd_sum, k_bwd_dm   sums over slices, then dM per head (sum over the batch in fixed order)
// Everything is in the log2 domain with the fp16 operands A' = alpha log2e W M and M' of the forward path.
// Key shifts: one scalar per slice, the forward path's running shift c*_p (the largest shift of slices 0..p),
// under which the slice's prefix state is stored and its keys are featurised in both tile kernels; the
// suffix sums bring the later slices' contributions down to it.  So the key logits may rise or fall along a
// sequence without limit; what has to fit the fp32 exponent range (about 2^100 between the smallest useful
// and the largest feature) is their spread inside one slice.
#include <cmath>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

constexpr int kT = 32;        // tokens per tile
constexpr int kF = 256;       // features
constexpr int kD = 64;        // d = r = dv
constexpr int LDX = 72;       // row pitch (16-bit elements) of token tiles with 64 columns
constexpr int LDP = 264;      // ... of token tiles with 256 columns, and of the [dv][F] state copies
constexpr int LDT = 40;       // ... of the 32 x 32 tiles
constexpr int LDN = 33;       // fp32 pitch of the N^T exchange tile
constexpr float kBigShift = 3.0e4f;  // a shift that sends exp2 to zero

typedef unsigned short us;

__device__ __forceinline__ f32x16 mm_bf16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&a), *reinterpret_cast<bf16x8*>(&b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mm_f16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<half8*>(&a), *reinterpret_cast<half8*>(&b), c, 0, 0, 0);
}
// Operand fragment of a 32x32x16 MFMA from a tile stored [row][k] with k contiguous: lane (l32, hf) takes
// the eight elements k0 + 8 hf + [0,8) of row r0 + l32.  Serves the A operand (row = output row) and the B
// operand (row = output column) alike.
__device__ __forceinline__ u32x4 ld_direct(const us* base, int ld, int r0, int k0, int lane) {
  return *reinterpret_cast<const u32x4*>(base + (r0 + lane % 32) * ld + k0 + 8 * (lane / 32));
}
// The same fragment from a tile stored [k][n] with n contiguous (the contraction index is the row): two
// transposing reads.  Within a group of 16 lanes, lane i points at row i / 4, columns 4 (i % 4) .. + 3 of a
// 4 x 16 patch and lane l receives column l of the four rows.
__device__ __forceinline__ u32x4 ld_tr(const us* base, int ld, int k0, int n0, int lane) {
  const int l16 = lane % 16, grp = lane / 16;
  const us* p = base + (k0 + 8 * (grp / 2) + l16 / 4) * ld + n0 + 16 * (grp % 2) + 4 * (l16 % 4);
  const u32x2 lo = lds_read_tr16(p);
  const u32x2 hi = lds_read_tr16(p + 4 * ld);
  return u32x4{lo[0], lo[1], hi[0], hi[1]};
}
__device__ __forceinline__ unsigned pack_f16(float a, float b) {
  fp16x2 h;
  h[0] = (__fp16)a;
  h[1] = (__fp16)b;
  return *reinterpret_cast<unsigned*>(&h);
}
__device__ __forceinline__ float bf_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
constexpr unsigned kOnes = 0x3f803f80u;

struct BwdSmem {
  // byte offsets; F = forward-order kernel, R = reverse-order kernel (same map, a few regions differ in use)
  static constexpr size_t al = 0;                                  // A' fp16 [256][LDX]
  static constexpr size_t st = al + (size_t)kF * LDX * 2;          // state copy bf16 [64][LDP]: S^T (F) / Rn^T (R)
  static constexpr size_t pq = st + (size_t)kD * LDP * 2;          // phi_Q tile [32][LDP] (R: later the logit gradients)
  static constexpr size_t pk = pq + (size_t)kT * LDP * 2;          // phi_K tile
  static constexpr size_t dl = pk + (size_t)kT * LDP * 2;          // F: logit gradients fp16 [32][LDP];  R: G2 = M'^T M' fp16 [64][LDX]
  static constexpr size_t xq = dl + (size_t)kT * LDP * 2;          // fp16 [32][LDX]
  static constexpr size_t xk = xq + (size_t)kT * LDX * 2;
  static constexpr size_t vt = xk + (size_t)kT * LDX * 2;          // bf16 [32][LDX]
  static constexpr size_t gr = vt + (size_t)kT * LDX * 2;          // raw dOut tile bf16
  static constexpr size_t gh = gr + (size_t)kT * LDX * 2;          // F: dOut / D (bf16)
  static constexpr size_t at = gh + (size_t)kT * LDX * 2;          // kernel-value tile bf16 [32][LDT]
  static constexpr size_t et = at + (size_t)kT * LDT * 2;          // E tile bf16 [32][LDT]
  static constexpr size_t nt = et + (size_t)kT * LDT * 2;          // F: N^T fp32 [64][LDN]; then the staging tile fp32 [32][64] of dQ (F), dV and dK (R)
  static constexpr size_t zs = nt + (size_t)kD * LDN * 4;          // F: z fp32 [256];  R: Rd fp32 [256]
  static constexpr size_t zb = zs + (size_t)kF * 4;                // F: z bf16 [256]
  static constexpr size_t mx = zb + (size_t)kF * 2;                // fp32 [8][32]: row maxima (F) / partial row sums (R)
  static constexpr size_t sc = mx + (size_t)8 * kT * 4;            // fp32 [8][32] per-token scalars
  static constexpr size_t total = sc + (size_t)8 * kT * 4;
};
static_assert(BwdSmem::total <= 160 * 1024, "backward tiles must fit the LDS of one CU");
static_assert((size_t)kD * LDX * 2 <= (size_t)kT * LDP * 2, "G2 must fit the region it borrows");

// Per-token scalar slots in BwdSmem::sc
enum { SC_NK = 0, SC_MU = 1, SC_DSUM = 2, SC_RHO = 3, SC_GDH = 4, SC_LAM = 5, SC_GD = 6, SC_S = 7 };

// The 32-token tiles of Q, K (converted to fp16), V and dOut (bf16; zero past the end): fetched into
// registers a tile ahead (tile_fetch), written to LDS when the previous tile is done with the buffers
// (tile_commit).  Threads 0..255 carry Q and V pieces, the others K and dOut pieces.
struct TileRegs {
  u32x4 x, y;
};
__device__ __forceinline__ TileRegs tile_fetch(const us* Qb, const us* Kb, const us* Vb, const us* Gb, int tok0, int L,
                                               int tid) {
  const int c = tid % 256, row = c / 8, ch = c % 8;
  const int tok = tok0 + row;
  const bool in = tok < L;
  const size_t off = (size_t)max(min(tok, L - 1), 0) * kD + 8 * ch;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  TileRegs r;
  if (tid < 256) {
    r.x = *reinterpret_cast<const u32x4*>(Qb + off);
    r.y = in ? *reinterpret_cast<const u32x4*>(Vb + off) : zero;
  } else {
    r.x = *reinterpret_cast<const u32x4*>(Kb + off);
    r.y = in ? *reinterpret_cast<const u32x4*>(Gb + off) : zero;
  }
  return r;
}
__device__ __forceinline__ void tile_commit(unsigned char* smem, const TileRegs& r, int tid) {
  const int c = tid % 256, row = c / 8, ch = c % 8;
  us* xdst = reinterpret_cast<us*>(smem + (tid < 256 ? BwdSmem::xq : BwdSmem::xk));
  us* ydst = reinterpret_cast<us*>(smem + (tid < 256 ? BwdSmem::vt : BwdSmem::gr));
  *reinterpret_cast<u32x4*>(xdst + row * LDX + 8 * ch) = bf16x8_to_f16x8(r.x);
  *reinterpret_cast<u32x4*>(ydst + row * LDX + 8 * ch) = r.y;
}

// A' of head h into LDS.
__device__ __forceinline__ void load_a(unsigned char* smem, const _Float16* Ah, int h, int tid) {
  us* Al = reinterpret_cast<us*>(smem + BwdSmem::al);
  const us* src = reinterpret_cast<const us*>(Ah) + (size_t)h * kF * kD;
#pragma unroll
  for (int u = 0; u < kF * kD / 8 / 512; ++u) {
    const int ci = tid + 512 * u, row = ci / 8, ch = ci % 8;
    *reinterpret_cast<u32x4*>(Al + row * LDX + 8 * ch) = *reinterpret_cast<const u32x4*>(src + (size_t)row * kD + 8 * ch);
  }
}

// Writes a wave's 32-feature block of a [feature][dv] fp32 state (two 32 x 32 accumulators: lane = value
// column, registers = features 8 a + 4 hf + j) as bf16 into the [dv][F] copy.
__device__ __forceinline__ void store_state_copy(us* St, const f32x16 (&S)[2], int wv, int lane) {
  const int l32 = lane % 32, hf = lane / 32;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const u32x2 w = {pack_bf16(S[db][4 * a], S[db][4 * a + 1]), pack_bf16(S[db][4 * a + 2], S[db][4 * a + 3])};
      *reinterpret_cast<u32x2*>(St + (32 * db + l32) * LDP + 32 * wv + 8 * a + 4 * hf) = w;
    }
}

// Gradient tiles (32 tokens x 64, fp32) leave through LDS: the waves that hold the accumulators write them
// to a staging tile, and after the next barrier all threads store full rows (16 bytes per lane, a row per
// 16 lanes), the rows past the end of the sequence left out.  (Stores straight from the accumulator layout
// need an address per row, which cost registers or spills.)
__device__ __forceinline__ void stage_tile(float* Ns, const f32x16& acc, float f, int cb, int lane) {
#pragma unroll
  for (int v = 0; v < 16; ++v) Ns[(8 * (v / 4) + 4 * (lane / 32) + (v % 4)) * kD + 32 * cb + lane % 32] = f * acc[v];
}
__device__ __forceinline__ void flush_tile(const float* Ns, float* dst, size_t row0, int nvalid, int tid) {
  const int row = tid / 16, ch = tid % 16;
  if (row < nvalid) *reinterpret_cast<f32x4*>(dst + (row0 + row) * kD + 4 * ch) = *reinterpret_cast<const f32x4*>(Ns + row * kD + 4 * ch);
}

// ---------------------------------------------------------------------------
// k_bwd_fwd
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(512, 1) void k_bwd_fwd(const us* __restrict__ Qg, const us* __restrict__ Kg,
                                                   const us* __restrict__ Vg, const us* __restrict__ Gg,
                                                   const _Float16* __restrict__ Ah, const float* __restrict__ nrm,
                                                   const float* __restrict__ Spre, const float* __restrict__ zpre,
                                                   const float* __restrict__ cpre, float* __restrict__ dQ,
                                                   float* __restrict__ lam, float* __restrict__ gdv,
                                                   float* __restrict__ dRn, float* __restrict__ dRd,
                                                   float* __restrict__ TQ, int H, int L, int P, int slice_len,
                                                   float inv_log2e) {
  using SM = BwdSmem;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  us* Al = reinterpret_cast<us*>(smem + SM::al);
  us* St = reinterpret_cast<us*>(smem + SM::st);
  us* PQ = reinterpret_cast<us*>(smem + SM::pq);
  us* PK = reinterpret_cast<us*>(smem + SM::pk);
  us* DL = reinterpret_cast<us*>(smem + SM::dl);
  us* Xq = reinterpret_cast<us*>(smem + SM::xq);
  us* Vt = reinterpret_cast<us*>(smem + SM::vt);
  us* Gr = reinterpret_cast<us*>(smem + SM::gr);
  us* Gh = reinterpret_cast<us*>(smem + SM::gh);
  us* At = reinterpret_cast<us*>(smem + SM::at);
  us* Et = reinterpret_cast<us*>(smem + SM::et);
  float* Nt = reinterpret_cast<float*>(smem + SM::nt);
  float* zs = reinterpret_cast<float*>(smem + SM::zs);
  us* zb = reinterpret_cast<us*>(smem + SM::zb);
  float* mx = reinterpret_cast<float*>(smem + SM::mx);
  float* sc = reinterpret_cast<float*>(smem + SM::sc);

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int bh = blockIdx.x / P, p = blockIdx.x % P;
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  if (tok_begin >= tok_end) return;
  const int ntile = (tok_end - tok_begin + kT - 1) / kT;
  const us* Qb = Qg + (size_t)bh * L * kD;
  const us* Kb = Kg + (size_t)bh * L * kD;
  const us* Vb = Vg + (size_t)bh * L * kD;
  const us* Gb = Gg + (size_t)bh * L * kD;
  const float c_ref = cpre[(size_t)bh * P + p];  // the running shift of this slice: its prefix state is expressed in it
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  load_a(smem, Ah, h, tid);
  // running state of this wave's 32 features: S [f][dv] (two value-column blocks), z (every column alike),
  // and the slice's contributions to Rn, Rd, T_Q
  // z (fp32 in LDS, feature tid of threads 0..255) and the slice's Rd (feature tid - 256 of the others,
  // in a register) are kept by the vector ALU: a column sum per tile
  f32x16 S[2], Rn[2], Tq[2];
  float rd_acc = 0.f;
  {
    const size_t sb = ((size_t)bh * P + p) * kF;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ft = 32 * wv + 8 * (v / 4) + 4 * hf + (v % 4);
        S[db][v] = Spre[(sb + ft) * kD + 32 * db + l32];
      }
    if (tid < kF) {
      const float z0 = zpre[sb + tid];
      zs[tid] = z0;
      zb[tid] = (us)(pack_bf16(z0, 0.f) & 0xffffu);
    }
  }
#pragma unroll
  for (int db = 0; db < 2; ++db) Rn[db] = Tq[db] = zero16;
  auto publish_state = [&]() { store_state_copy(St, S, wv, lane); };
  publish_state();
  __syncthreads();

  TileRegs nxt = tile_fetch(Qb, Kb, Vb, Gb, tok_begin, L, tid);
  float nk_nxt = (tid < kT && tok_begin + tid < L) ? nrm[(size_t)bh * L + tok_begin + tid] : kBigShift;
  for (int t = 0; t < ntile; ++t) {
    const int tok0 = tok_begin + t * kT;
    // ---- stage 0: this tile into LDS, the next one on its way -------------------------------------
    tile_commit(smem, nxt, tid);
    if (dQ != nullptr && t > 0) flush_tile(Nt, dQ, (size_t)bh * L + tok0 - kT, kT, tid);  // the previous tile's dQ
    if (tid < kT) sc[SC_NK * kT + tid] = nk_nxt;
    if (t + 1 < ntile) {
      nxt = tile_fetch(Qb, Kb, Vb, Gb, tok0 + kT, L, tid);
      nk_nxt = (tid < kT && tok0 + kT + tid < L) ? nrm[(size_t)bh * L + tok0 + kT + tid] : kBigShift;
    }
    __syncthreads();
    // ---- stage 1: projections, features ---------------------------------------------------------
    const us* Xk = reinterpret_cast<const us*>(smem + SM::xk);
    f32x16 uq = zero16, uk = zero16;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const u32x4 af = ld_direct(Al, LDX, 32 * wv, 16 * s, lane);  // A' rows of this wave's features
      uq = mm_f16(af, ld_direct(Xq, LDX, 0, 16 * s, lane), uq);
      uk = mm_f16(af, ld_direct(Xk, LDX, 0, 16 * s, lane), uk);
    }
    {
      const float sub = sc[SC_NK * kT + l32] + c_ref;
      float m0 = uq[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) m0 = fmaxf(m0, uq[v]);
      m0 = fmaxf(m0, __shfl_xor(m0, 32, 64));
      if (hf == 0) mx[wv * kT + l32] = m0;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const u32x2 w = {pack_bf16(fast_exp2(uk[4 * a] - sub), fast_exp2(uk[4 * a + 1] - sub)),
                         pack_bf16(fast_exp2(uk[4 * a + 2] - sub), fast_exp2(uk[4 * a + 3] - sub))};
        *reinterpret_cast<u32x2*>(PK + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = w;
      }
    }
    __syncthreads();
    {
      float mu = mx[l32];
#pragma unroll
      for (int w = 1; w < 8; ++w) mu = fmaxf(mu, mx[w * kT + l32]);
      if (wv == 0 && hf == 0) sc[SC_MU * kT + l32] = mu;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const u32x2 w = {pack_bf16(fast_exp2(uq[4 * a] - mu), fast_exp2(uq[4 * a + 1] - mu)),
                         pack_bf16(fast_exp2(uq[4 * a + 2] - mu), fast_exp2(uq[4 * a + 3] - mu))};
        *reinterpret_cast<u32x2*>(PQ + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = w;
      }
    }
    __syncthreads();
    // ---- stage 2: kernel values of the tile, At[i][l] = phi_Q,i . phi_K,l for l <= i ---------------
    if (wv == 0) {
      f32x16 acc = zero16;  // rows l, columns i
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) acc = mm_bf16(ld_direct(PK, LDP, 0, 16 * s, lane), ld_direct(PQ, LDP, 0, 16 * s, lane), acc);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = (8 * a + 4 * hf + j <= l32) ? acc[4 * a + j] : 0.f;
        const u32x2 w = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3])};
        *reinterpret_cast<u32x2*>(At + l32 * LDT + 8 * a + 4 * hf) = w;
      }
    }
    __syncthreads();
    // ---- stage 3: numerator N^T[dv][i] (waves 0, 1) and denominator (wave 2) ------------------------
    if (wv < 2) {
      f32x16 acc = zero16;  // rows dv, columns i
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) acc = mm_bf16(ld_direct(St, LDP, 32 * wv, 16 * s, lane), ld_direct(PQ, LDP, 0, 16 * s, lane), acc);
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) acc = mm_bf16(ld_tr(Vt, LDX, 16 * s, 32 * wv, lane), ld_direct(At, LDT, 0, 16 * s, lane), acc);
#pragma unroll
      for (int v = 0; v < 16; ++v) Nt[(32 * wv + 8 * (v / 4) + 4 * hf + (v % 4)) * LDN + l32] = acc[v];
    } else if (wv == 2) {
      f32x16 acc = zero16;  // every row: the denominator of column i
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) {
        const u32x4 zf = *reinterpret_cast<const u32x4*>(zb + 16 * s + 8 * hf);
        acc = mm_bf16(zf, ld_direct(PQ, LDP, 0, 16 * s, lane), acc);
      }
      const u32x4 ones = {kOnes, kOnes, kOnes, kOnes};
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) acc = mm_bf16(ones, ld_direct(At, LDT, 0, 16 * s, lane), acc);
      if (hf == 0) sc[SC_DSUM * kT + l32] = acc[0];
    }
    __syncthreads();
    // ---- per-token scalars: rho = 1 / D, gd, lambda; the scaled dOut tile ----------------------------
    {
      const int i = tid / 16, q = tid % 16;
      const bool valid = tok0 + i < L;
      const float dsum = sc[SC_DSUM * kT + i];
      const float rho = valid ? 1.f / dsum : 0.f;
      const u32x2 gw = *reinterpret_cast<const u32x2*>(Gr + i * LDX + 4 * q);
      // dOut / D is rounded to bf16 for the MFMAs; gd is formed from the rounded values, so that
      // E_il = Ghat_i . v_l + gdhat_i is exactly Ghat_i . (v_l - out_i) and cancels where it should
      const u32x2 w = {pack_bf16(rho * bf_lo(gw[0]), rho * bf_hi(gw[0])), pack_bf16(rho * bf_lo(gw[1]), rho * bf_hi(gw[1]))};
      *reinterpret_cast<u32x2*>(Gh + i * LDX + 4 * q) = w;
      float dot = bf_lo(w[0]) * Nt[(4 * q) * LDN + i] + bf_hi(w[0]) * Nt[(4 * q + 1) * LDN + i] +
                  bf_lo(w[1]) * Nt[(4 * q + 2) * LDN + i] + bf_hi(w[1]) * Nt[(4 * q + 3) * LDN + i];
      dot += __shfl_xor(dot, 8, 64);
      dot += __shfl_xor(dot, 4, 64);
      dot += __shfl_xor(dot, 2, 64);
      dot += __shfl_xor(dot, 1, 64);   // = Ghat_i . N_i
      float draw = bf_lo(gw[0]) * Nt[(4 * q) * LDN + i] + bf_hi(gw[0]) * Nt[(4 * q + 1) * LDN + i] +
                   bf_lo(gw[1]) * Nt[(4 * q + 2) * LDN + i] + bf_hi(gw[1]) * Nt[(4 * q + 3) * LDN + i];
      draw += __shfl_xor(draw, 8, 64);
      draw += __shfl_xor(draw, 4, 64);
      draw += __shfl_xor(draw, 2, 64);
      draw += __shfl_xor(draw, 1, 64);  // = G_i . N_i (the reverse pass works with the unscaled dOut)
      if (q == 0) {
        sc[SC_RHO * kT + i] = rho;
        sc[SC_GDH * kT + i] = -rho * dot;
        if (valid) {
          lam[(size_t)bh * L + tok0 + i] = sc[SC_MU * kT + i] + __builtin_log2f(dsum);
          gdv[(size_t)bh * L + tok0 + i] = -rho * draw;
        }
      }
    }
    __syncthreads();
    // ---- stage 4: Et[i][l] = (G_i . v_l + gd_i) / D_i for l <= i --------------------------------------
    if (wv == 0) {
      f32x16 acc = zero16;  // rows l, columns i
#pragma unroll
      for (int s = 0; s < kD / 16; ++s) acc = mm_bf16(ld_direct(Vt, LDX, 0, 16 * s, lane), ld_direct(Gh, LDX, 0, 16 * s, lane), acc);
      const float gd = sc[SC_GDH * kT + l32];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = (8 * a + 4 * hf + j <= l32) ? acc[4 * a + j] + gd : 0.f;
        const u32x2 w = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3])};
        *reinterpret_cast<u32x2*>(Et + l32 * LDT + 8 * a + 4 * hf) = w;
      }
    }
    __syncthreads();
    // ---- stage 5: dlogit_Q^T[f][i] = phi_Q ( S Ghat_i + z gdhat_i + sum_{l<=i} E_il phi_K,l ) ----------
    {
      f32x16 acc = zero16;  // rows f (this wave's 32), columns i
#pragma unroll
      for (int s = 0; s < kD / 16; ++s) acc = mm_bf16(ld_tr(St, LDP, 16 * s, 32 * wv, lane), ld_direct(Gh, LDX, 0, 16 * s, lane), acc);
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) acc = mm_bf16(ld_tr(PK, LDP, 16 * s, 32 * wv, lane), ld_direct(Et, LDT, 0, 16 * s, lane), acc);
      const float gd = sc[SC_GDH * kT + l32];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        // z as the denominator saw it (rounded to bf16): with the same S, z and features in out_i and here,
        // the terms G_i . (v_l - out_i) cancel as they do in exact arithmetic
        const u32x2 zw = *reinterpret_cast<const u32x2*>(zb + 32 * wv + 8 * a + 4 * hf);
        const u32x2 pw = *reinterpret_cast<const u32x2*>(PQ + l32 * LDP + 32 * wv + 8 * a + 4 * hf);
        const float d0 = bf_lo(pw[0]) * fmaf(bf_lo(zw[0]), gd, acc[4 * a]);
        const float d1 = bf_hi(pw[0]) * fmaf(bf_hi(zw[0]), gd, acc[4 * a + 1]);
        const float d2 = bf_lo(pw[1]) * fmaf(bf_lo(zw[1]), gd, acc[4 * a + 2]);
        const float d3 = bf_hi(pw[1]) * fmaf(bf_hi(zw[1]), gd, acc[4 * a + 3]);
        const u32x2 w = {pack_f16(d0, d1), pack_f16(d2, d3)};
        *reinterpret_cast<u32x2*>(DL + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = w;
      }
    }
    __syncthreads();
    // ---- stage 6: dQ, and the state updates -----------------------------------------------------------
    if (wv < 2 && dQ != nullptr) {
      f32x16 acc = zero16;  // rows i, columns d (32 wv + l32)
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) acc = mm_f16(ld_direct(DL, LDP, 0, 16 * s, lane), ld_tr(Al, LDX, 16 * s, 32 * wv, lane), acc);
      stage_tile(Nt, acc, inv_log2e, wv, lane);
    }
#pragma unroll
    for (int s = 0; s < kT / 16; ++s) {
      const u32x4 dlf = ld_tr(DL, LDP, 16 * s, 32 * wv, lane);
      const u32x4 pkf = ld_tr(PK, LDP, 16 * s, 32 * wv, lane);
      const u32x4 pqf = ld_tr(PQ, LDP, 16 * s, 32 * wv, lane);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        Tq[db] = mm_f16(dlf, ld_tr(Xq, LDX, 16 * s, 32 * db, lane), Tq[db]);
        S[db] = mm_bf16(pkf, ld_tr(Vt, LDX, 16 * s, 32 * db, lane), S[db]);
        Rn[db] = mm_bf16(pqf, ld_tr(Gh, LDX, 16 * s, 32 * db, lane), Rn[db]);
      }
    }
    if (tid < kF) {  // z_f += sum_l phi_K,lf
      float a = 0.f;
#pragma unroll
      for (int l = 0; l < kT; ++l) a += __uint_as_float((unsigned)PK[l * LDP + tid] << 16);
      const float z1 = zs[tid] + a;
      zs[tid] = z1;
      zb[tid] = (us)(pack_bf16(z1, 0.f) & 0xffffu);
    } else {         // Rd_f += sum_i phi_Q,if gdhat_i
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < kT; ++i) a = fmaf(__uint_as_float((unsigned)PQ[i * LDP + tid - kF] << 16), sc[SC_GDH * kT + i], a);
      rd_acc += a;
    }
    publish_state();
    __syncthreads();
  }
  if (dQ != nullptr) flush_tile(Nt, dQ, (size_t)bh * L + tok_begin + (ntile - 1) * kT, min(kT, L - (tok_begin + (ntile - 1) * kT)), tid);
  // ---- the slice's contributions ---------------------------------------------------------------------
  const size_t ob = ((size_t)bh * P + p) * kF;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int ft = 32 * wv + 8 * (v / 4) + 4 * hf + (v % 4);
      dRn[(ob + ft) * kD + 32 * db + l32] = Rn[db][v];
      TQ[(ob + ft) * kD + 32 * db + l32] = Tq[db][v];
    }
  if (tid >= kF) dRd[ob + tid - kF] = rd_acc;
}

// ---------------------------------------------------------------------------
// k_bwd_suffix: Rsuf_p = sum_{p' > p} 2^(c*_p - c*_p') dR_p' (p' descending: fixed order), separate output.
// The contribution of slice p' was formed with denominators in the scale of its own running shift c*_p', and
// meets key features of slice p, which are in the scale of c*_p <= c*_p': the factor (at most one) brings it
// there.  One thread per four state entries; the Rd vector rides at the end.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bwd_suffix(const float* __restrict__ dRn, const float* __restrict__ dRd,
                                                    const float* __restrict__ cpre, float* __restrict__ Rn,
                                                    float* __restrict__ Rd, int P, long long BH) {
  // four consecutive entries per thread; per (b,h) the kF x kD entries of Rn, then the kF of Rd
  const long long per4 = ((long long)kF * kD + kF) / 4;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= BH * per4) return;
  const long long bh = idx / per4, e = 4 * (idx % per4);
  const bool isn = e < (long long)kF * kD;
  const float* src = isn ? dRn + (size_t)bh * P * kF * kD + e : dRd + (size_t)bh * P * kF + (e - (long long)kF * kD);
  float* dst = isn ? Rn + (size_t)bh * P * kF * kD + e : Rd + (size_t)bh * P * kF + (e - (long long)kF * kD);
  const size_t pitch = isn ? (size_t)kF * kD : (size_t)kF;
  const float* cb = cpre + (size_t)bh * P;
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  float c_later = 0.f;  // shift of the slice handled last
  for (int p0 = P - 1; p0 >= 0; p0 -= 8) {   // eight slices' loads in flight, then the (ordered) running sums
    f32x4 v[8];
    float c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p0 - u >= 0) {
        v[u] = *reinterpret_cast<const f32x4*>(src + (size_t)(p0 - u) * pitch);
        c[u] = cb[p0 - u];
      }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p0 - u >= 0) {
        if (p0 - u < P - 1) run *= fast_exp2(c[u] - c_later);
        c_later = c[u];
        *reinterpret_cast<f32x4*>(dst + (size_t)(p0 - u) * pitch) = run;
        run += v[u];
      }
  }
}

// ---------------------------------------------------------------------------
// k_bwd_rev
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(512, 1) void k_bwd_rev(const us* __restrict__ Qg, const us* __restrict__ Kg,
                                                   const us* __restrict__ Vg, const us* __restrict__ Gg,
                                                   const _Float16* __restrict__ Ah, const _Float16* __restrict__ Mh,
                                                   const float* __restrict__ nrm, const float* __restrict__ cpre,
                                                   const float* __restrict__ lam, const float* __restrict__ gdv,
                                                   const float* __restrict__ Rsn, const float* __restrict__ Rsd,
                                                   float* __restrict__ dK, float* __restrict__ dV,
                                                   const float* __restrict__ TQ, float* __restrict__ TK,
                                                   float* __restrict__ RM, int H, int L, int P, int slice_len,
                                                   float inv_log2e) {
  using SM = BwdSmem;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  us* Al = reinterpret_cast<us*>(smem + SM::al);
  us* Rt = reinterpret_cast<us*>(smem + SM::st);
  us* PQ = reinterpret_cast<us*>(smem + SM::pq);
  us* DL = PQ;  // the logit gradients take the place of phihat_Q (each wave owns its 32 feature columns of both)
  us* PK = reinterpret_cast<us*>(smem + SM::pk);
  us* G2 = reinterpret_cast<us*>(smem + SM::dl);
  us* Xq = reinterpret_cast<us*>(smem + SM::xq);
  us* Xk = reinterpret_cast<us*>(smem + SM::xk);
  us* Vt = reinterpret_cast<us*>(smem + SM::vt);
  us* Gr = reinterpret_cast<us*>(smem + SM::gr);
  us* At = reinterpret_cast<us*>(smem + SM::at);   // AtT[l][i]
  us* Et = reinterpret_cast<us*>(smem + SM::et);   // ET[l][i]
  float* Ns = reinterpret_cast<float*>(smem + SM::nt);  // staging tile of dV, then of dK
  float* rd = reinterpret_cast<float*>(smem + SM::zs);
  float* sp = reinterpret_cast<float*>(smem + SM::mx);
  float* sc = reinterpret_cast<float*>(smem + SM::sc);

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int bh = blockIdx.x / P, p = blockIdx.x % P;
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  if (tok_begin >= tok_end) return;
  const int ntile = (tok_end - tok_begin + kT - 1) / kT;
  const us* Qb = Qg + (size_t)bh * L * kD;
  const us* Kb = Kg + (size_t)bh * L * kD;
  const us* Vb = Vg + (size_t)bh * L * kD;
  const us* Gb = Gg + (size_t)bh * L * kD;
  const float c_ref = cpre[(size_t)bh * P + p];  // keys of this slice are featurised under its own running shift
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  load_a(smem, Ah, h, tid);
  {  // M' of the head into the phi_K region for a moment: G2 = M'^T M' (= alpha^2 log2e/2 M^T M)
    const us* src = reinterpret_cast<const us*>(Mh) + (size_t)h * kD * kD;
    const int row = tid / 8, ch = tid % 8;
    *reinterpret_cast<u32x4*>(PK + row * LDX + 8 * ch) = *reinterpret_cast<const u32x4*>(src + (size_t)row * kD + 8 * ch);
  }
  __syncthreads();
  if (wv < 4) {
    const int eb = wv / 2, db = wv % 2;
    f32x16 acc = zero16;  // rows e, columns d
#pragma unroll
    for (int s = 0; s < kD / 16; ++s) acc = mm_f16(ld_tr(PK, LDX, 16 * s, 32 * eb, lane), ld_tr(PK, LDX, 16 * s, 32 * db, lane), acc);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      fp16x2 hv2;
      hv2[0] = (__fp16)acc[v];
      hv2[1] = (__fp16)0.f;
      G2[(32 * eb + 8 * (v / 4) + 4 * hf + (v % 4)) * LDX + 32 * db + l32] = (us)(*reinterpret_cast<unsigned*>(&hv2) & 0xffffu);
    }
  }
  // running suffix state of this wave's 32 features, the slice's T_K; Rm block of waves 4..7
  f32x16 Rn[2], Tk[2], Rm;
  float rd_new = 0.f;  // threads 256..511: Rd of feature tid - 256 after the current tile (published at the end of the tile)
  {
    const size_t sb = ((size_t)bh * P + p) * kF;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ft = 32 * wv + 8 * (v / 4) + 4 * hf + (v % 4);
        Rn[db][v] = Rsn[(sb + ft) * kD + 32 * db + l32];
      }
    if (tid >= kF) rd_new = Rsd[sb + tid - kF];
  }
  {  // T of the slice: the query half comes from the forward-order pass, the key half is added here
    const size_t sb = ((size_t)bh * P + p) * kF;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) Tk[db][v] = TQ[(sb + 32 * wv + 8 * (v / 4) + 4 * hf + (v % 4)) * kD + 32 * db + l32];
  }
  Rm = zero16;
  auto publish_state = [&]() {
    store_state_copy(Rt, Rn, wv, lane);
    if (tid >= kF) rd[tid - kF] = rd_new;
  };
  publish_state();
  __syncthreads();

  auto fetch_scalars = [&](int tk0, float& a, float& b, float& c) {
    const bool valid = tid < kT && tk0 + tid < L;
    a = valid ? nrm[(size_t)bh * L + tk0 + tid] : kBigShift;
    b = valid ? lam[(size_t)bh * L + tk0 + tid] : kBigShift;
    c = valid ? gdv[(size_t)bh * L + tk0 + tid] : 0.f;
  };
  TileRegs nxt = tile_fetch(Qb, Kb, Vb, Gb, tok_begin + (ntile - 1) * kT, L, tid);
  float s_nk, s_lam, s_gd;
  fetch_scalars(tok_begin + (ntile - 1) * kT, s_nk, s_lam, s_gd);
  for (int t = ntile - 1; t >= 0; --t) {
    const int tok0 = tok_begin + t * kT;
    // ---- stage 0: this tile into LDS, the next one (towards the start of the slice) on its way --------
    tile_commit(smem, nxt, tid);
    if (dK != nullptr && t < ntile - 1) flush_tile(Ns, dK, (size_t)bh * L + tok0 + kT, min(kT, L - (tok0 + kT)), tid);  // the previous tile's dK
    if (tid < kT) {
      sc[SC_NK * kT + tid] = s_nk;
      sc[SC_LAM * kT + tid] = s_lam;
      sc[SC_GD * kT + tid] = s_gd;
    }
    if (t > 0) {
      nxt = tile_fetch(Qb, Kb, Vb, Gb, tok0 - kT, L, tid);
      fetch_scalars(tok0 - kT, s_nk, s_lam, s_gd);
    }
    lds_barrier();
    // ---- stage 1: phihat_Q = exp2(u - lambda), phi_K ------------------------------------------------
    {
      f32x16 uq = zero16, uk = zero16;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const u32x4 af = ld_direct(Al, LDX, 32 * wv, 16 * s, lane);
        uq = mm_f16(af, ld_direct(Xq, LDX, 0, 16 * s, lane), uq);
        uk = mm_f16(af, ld_direct(Xk, LDX, 0, 16 * s, lane), uk);
      }
      const float subk = sc[SC_NK * kT + l32] + c_ref;
      const float subq = sc[SC_LAM * kT + l32];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const u32x2 wk = {pack_bf16(fast_exp2(uk[4 * a] - subk), fast_exp2(uk[4 * a + 1] - subk)),
                          pack_bf16(fast_exp2(uk[4 * a + 2] - subk), fast_exp2(uk[4 * a + 3] - subk))};
        *reinterpret_cast<u32x2*>(PK + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = wk;
        const u32x2 wq = {pack_bf16(fast_exp2(uq[4 * a] - subq), fast_exp2(uq[4 * a + 1] - subq)),
                          pack_bf16(fast_exp2(uq[4 * a + 2] - subq), fast_exp2(uq[4 * a + 3] - subq))};
        *reinterpret_cast<u32x2*>(PQ + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = wq;
      }
    }
    lds_barrier();
    // ---- stage 2: AtT[l][i] = a_il / D_i (wave 0), ET[l][i] = G_i . v_l + gd_i (wave 1), i >= l --------
    if (wv == 0) {
      f32x16 acc = zero16;  // rows i, columns l
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) acc = mm_bf16(ld_direct(PQ, LDP, 0, 16 * s, lane), ld_direct(PK, LDP, 0, 16 * s, lane), acc);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = (8 * a + 4 * hf + j >= l32) ? acc[4 * a + j] : 0.f;
        const u32x2 w = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3])};
        *reinterpret_cast<u32x2*>(At + l32 * LDT + 8 * a + 4 * hf) = w;
      }
    } else if (wv == 1) {
      f32x16 acc = zero16;  // rows i, columns l
#pragma unroll
      for (int s = 0; s < kD / 16; ++s) acc = mm_bf16(ld_direct(Gr, LDX, 0, 16 * s, lane), ld_direct(Vt, LDX, 0, 16 * s, lane), acc);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const f32x4 g4 = *reinterpret_cast<const f32x4*>(sc + SC_GD * kT + 8 * a + 4 * hf);
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = (8 * a + 4 * hf + j >= l32) ? acc[4 * a + j] + g4[j] : 0.f;
        const u32x2 w = {pack_bf16(e[0], e[1]), pack_bf16(e[2], e[3])};
        *reinterpret_cast<u32x2*>(Et + l32 * LDT + 8 * a + 4 * hf) = w;
      }
    } else if (wv >= 4) {  // Rd_f += sum_i phihat_Q,if gd_i (before the logit gradients take phihat_Q's place)
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < kT; ++i) a = fmaf(__uint_as_float((unsigned)PQ[i * LDP + tid - kF] << 16), sc[SC_GD * kT + i], a);
      rd_new += a;
    }
    lds_barrier();
    // ---- stage 3: dV (waves 0, 1); dlogit_K^T[f][l]; the suffix state takes the tile's queries -----------
    if (wv < 2 && dV != nullptr) {
      f32x16 acc = zero16;  // rows l, columns dv (32 wv + l32)
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) acc = mm_bf16(ld_direct(PK, LDP, 0, 16 * s, lane), ld_direct(Rt, LDP, 32 * wv, 16 * s, lane), acc);
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) acc = mm_bf16(ld_direct(At, LDT, 0, 16 * s, lane), ld_tr(Gr, LDX, 16 * s, 32 * wv, lane), acc);
      stage_tile(Ns, acc, 1.f, wv, lane);
    }
    {
      f32x16 acc = zero16;  // rows f (this wave's 32), columns l
#pragma unroll
      for (int s = 0; s < kD / 16; ++s) acc = mm_bf16(ld_tr(Rt, LDP, 16 * s, 32 * wv, lane), ld_direct(Vt, LDX, 0, 16 * s, lane), acc);
      u32x4 pqf[kT / 16];
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) {
        pqf[s] = ld_tr(PQ, LDP, 16 * s, 32 * wv, lane);
        acc = mm_bf16(pqf[s], ld_direct(Et, LDT, 0, 16 * s, lane), acc);
      }
      // the suffix state takes this tile's queries (all reads of phihat_Q are done before DL overwrites it)
#pragma unroll
      for (int s = 0; s < kT / 16; ++s)
#pragma unroll
        for (int db = 0; db < 2; ++db) Rn[db] = mm_bf16(pqf[s], ld_tr(Gr, LDX, 16 * s, 32 * db, lane), Rn[db]);
      float ssum = 0.f;
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const f32x4 r4 = *reinterpret_cast<const f32x4*>(rd + 32 * wv + 8 * a + 4 * hf);
        const u32x2 pw = *reinterpret_cast<const u32x2*>(PK + l32 * LDP + 32 * wv + 8 * a + 4 * hf);
        const float d0 = bf_lo(pw[0]) * (acc[4 * a] + r4[0]);
        const float d1 = bf_hi(pw[0]) * (acc[4 * a + 1] + r4[1]);
        const float d2 = bf_lo(pw[1]) * (acc[4 * a + 2] + r4[2]);
        const float d3 = bf_hi(pw[1]) * (acc[4 * a + 3] + r4[3]);
        ssum += (d0 + d1) + (d2 + d3);
        const u32x2 w = {pack_f16(d0, d1), pack_f16(d2, d3)};
        *reinterpret_cast<u32x2*>(DL + l32 * LDP + 32 * wv + 8 * a + 4 * hf) = w;
      }
      ssum += __shfl_xor(ssum, 32, 64);
      if (hf == 0) sp[wv * kT + l32] = ssum;
    }
    lds_barrier();
    // ---- stage 4: s_l; dK; T_K; Rm; publish the new suffix state -----------------------------------------
    if (tid < kT) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) s += sp[w * kT + tid];
      sc[SC_S * kT + tid] = s;
    }
    if (dV != nullptr) flush_tile(Ns, dV, (size_t)bh * L + tok0, min(kT, L - tok0), tid);
    lds_barrier();
    if (wv < 2 && dK != nullptr) {
      f32x16 acc = zero16, acc2 = zero16;  // rows l, columns d (32 wv + l32)
#pragma unroll 4
      for (int s = 0; s < kF / 16; ++s) {
        acc = mm_f16(ld_direct(DL, LDP, 0, 16 * s, lane), ld_tr(Al, LDX, 16 * s, 32 * wv, lane), acc);
      }
#pragma unroll
      for (int s = 0; s < kD / 16; ++s) acc2 = mm_f16(ld_direct(Xk, LDX, 0, 16 * s, lane), ld_direct(G2, LDX, 32 * wv, 16 * s, lane), acc2);
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] -= 2.f * sc[SC_S * kT + 8 * (v / 4) + 4 * hf + (v % 4)] * acc2[v];
      stage_tile(Ns, acc, inv_log2e, wv, lane);
    }
#pragma unroll
    for (int s = 0; s < kT / 16; ++s) {
      const u32x4 dlf = ld_tr(DL, LDP, 16 * s, 32 * wv, lane);
#pragma unroll
      for (int db = 0; db < 2; ++db) Tk[db] = mm_f16(dlf, ld_tr(Xk, LDX, 16 * s, 32 * db, lane), Tk[db]);
    }
    if (wv >= 4) {
      const int eb = (wv - 4) / 2, db = (wv - 4) % 2;
#pragma unroll
      for (int s = 0; s < kT / 16; ++s) {
        u32x4 xa = ld_tr(Xk, LDX, 16 * s, 32 * eb, lane);  // k_l[e] for l = 16 s + 8 hf + [0,8): scale by s_l
        const float* sl = sc + SC_S * kT + 16 * s + 8 * hf;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          unsigned wq = xa[q];
          fp16x2 hv2 = *reinterpret_cast<fp16x2*>(&wq);
          xa[q] = pack_f16((float)hv2[0] * sl[2 * q], (float)hv2[1] * sl[2 * q + 1]);
        }
        Rm = mm_f16(xa, ld_tr(Xk, LDX, 16 * s, 32 * db, lane), Rm);
      }
    }
    publish_state();
    lds_barrier();
  }
  if (dK != nullptr) flush_tile(Ns, dK, (size_t)bh * L + tok_begin, min(kT, L - tok_begin), tid);
  const size_t ob = ((size_t)bh * P + p) * kF;
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int ft = 32 * wv + 8 * (v / 4) + 4 * hf + (v % 4);
      TK[(ob + ft) * kD + 32 * db + l32] = Tk[db][v];
    }
  if (wv >= 4) {
    const int eb = (wv - 4) / 2, db = (wv - 4) % 2;
    const size_t rb = ((size_t)bh * P + p) * kD;
#pragma unroll
    for (int v = 0; v < 16; ++v) RM[(rb + 32 * eb + 8 * (v / 4) + 4 * hf + (v % 4)) * kD + 32 * db + l32] = Rm[v];
  }
}

// ---------------------------------------------------------------------------
// k_bwd_sum: per head, Tsum[h] = sum over batch entries and slices of the slice matrices T (queries and keys
// together), Rmsum[h] likewise; (b, p) ascending: fixed order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bwd_sum(const float* __restrict__ T, const float* __restrict__ RM,
                                                 float* __restrict__ Tsum, float* __restrict__ Rmsum, int B, int H, int P) {
  // four consecutive entries per thread; per head the kF x kD entries of T, then the kD x kD of Rm
  const long long per4 = ((long long)kF * kD + kD * kD) / 4;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)H * per4) return;
  const int h = (int)(idx / per4);
  const long long e = 4 * (idx % per4);
  const bool ist = e < (long long)kF * kD;
  const size_t pitch = ist ? (size_t)kF * kD : (size_t)kD * kD;
  const float* src = ist ? T + e : RM + (e - (long long)kF * kD);
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  const int n = B * P;   // slice s = b P + p of head h lies at ((b H + h) P + p) pitch
  for (int s0 = 0; s0 < n; s0 += 8) {
    f32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int sidx = s0 + u;
      if (sidx < n) v[u] = *reinterpret_cast<const f32x4*>(src + (((size_t)(sidx / P) * H + h) * P + sidx % P) * pitch);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < n) run += v[u];
  }
  float* dst = ist ? Tsum + (size_t)h * kF * kD + e : Rmsum + (size_t)h * kD * kD + (e - (long long)kF * kD);
  *reinterpret_cast<f32x4*>(dst) = run;
}

// ---------------------------------------------------------------------------
// k_bwd_dm: dM[h][r][d] = alpha sum_j W[h][j][r] Tsum[h][j][d] - alpha^2 sum_e M[h][r][e] Rmsum[h][e][d].
// One block per (h, four rows r): thread (r, d).  The four columns of W and rows of M go to LDS first (the
// strided reads once, together); the 320 terms of a thread are then read sixteen at a time.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bwd_dm(const float* __restrict__ Tsum, const float* __restrict__ Rmsum,
                                                const float* __restrict__ M, const float* __restrict__ W,
                                                float* __restrict__ dM, int H, int w_shared, float alpha) {
  __shared__ float Ws[kF * 4];
  __shared__ float Ms[4 * kD];
  const int h = blockIdx.x / (kD / 4), r0 = 4 * (blockIdx.x % (kD / 4));
  const int rr = threadIdx.x / kD, d = threadIdx.x % kD;
  const float* Wh = W + (w_shared ? 0 : (size_t)h * kF * kD);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = threadIdx.x + 256 * u;   // (j, c): W[j][r0 + c]
    Ws[i] = Wh[(size_t)(i / 4) * kD + r0 + i % 4];
  }
  Ms[threadIdx.x] = M[((size_t)h * kD + r0 + rr) * kD + d];
  __syncthreads();
  const float* Tp = Tsum + (size_t)h * kF * kD + d;
  const float* Rp = Rmsum + (size_t)h * kD * kD + d;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 < kF; j0 += 16) {
    float t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = Tp[(size_t)(j0 + u) * kD];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u % 4] = fmaf(Ws[(j0 + u) * 4 + rr], t[u], acc[u % 4]);
  }
  float acc2[4] = {0.f, 0.f, 0.f, 0.f};
  for (int e0 = 0; e0 < kD; e0 += 16) {
    float t[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) t[u] = Rp[(size_t)(e0 + u) * kD];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc2[u % 4] = fmaf(Ms[rr * kD + e0 + u], t[u], acc2[u % 4]);
  }
  dM[((size_t)h * kD + r0 + rr) * kD + d] =
      alpha * ((acc[0] + acc[1]) + (acc[2] + acc[3])) - alpha * alpha * ((acc2[0] + acc2[1]) + (acc2[2] + acc2[3]));
}

}  // namespace

bool fused_bwd_supported(const Problem& pb, bool causal) {
  const dark_params& p = pb.p;
  return causal && p.io_dtype == DARK_BF16 && p.d == 64 && p.r == 64 && p.dv == 64 && p.m == 256;
}

dark_status fused_attn_bwd(const Problem& pb, Arena& ar, const void* Q, const void* K, const void* V, const float* M,
                           const float* W, const void* dOut, float* dQ, float* dK, float* dV, float* dM, float* dW) {
  const dark_params& p = pb.p;
  const long long BH = pb.BH();
  int P, sl;
  causal_slices(pb, &P, &sl);

  const size_t nstate = (size_t)BH * P * kF;
  // operand copies, key norms and prefix states: from the forward's hand-over buffer when the caller has one
  Arena sv(pb.saved, pb.saved_bytes);
  const bool handover = pb.saved_mode == 2 && ar.base != nullptr;
  const CausalKeep kp = take_causal_keep(handover ? sv : ar, pb, P);
  _Float16 *Ah = kp.Ah, *Mh = kp.Mh;
  float *Spre = kp.Spre, *zpre = kp.zpre, *cpre = kp.cpre, *nrm = kp.nrm;
  unsigned short* Spart = ar.take<unsigned short>(nstate * kD);
  float* zpart = ar.take<float>(nstate);
  float* cpart = ar.take<float>(nstate);
  float* lam = ar.take<float>((size_t)BH * p.L);
  float* gdv = ar.take<float>((size_t)BH * p.L);
  float* dRn = ar.take<float>(nstate * kD);
  float* dRd = ar.take<float>(nstate);
  float* Rsn = ar.take<float>(nstate * kD);
  float* Rsd = ar.take<float>(nstate);
  float* TQ = ar.take<float>(nstate * kD);
  float* TK = ar.take<float>(nstate * kD);
  float* RM = ar.take<float>((size_t)BH * P * kD * kD);
  float* Tsum = ar.take<float>((size_t)p.H * kF * kD);
  float* Rmsum = ar.take<float>((size_t)p.H * kD * kD);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow || sv.overflow) return DARK_EWORKSPACE;

  if (!handover) {
    DARK_TRY(fused_launch_prep(pb, M, W, Ah, Mh));
    DARK_TRY(fused_causal_states64(pb, K, V, Ah, Mh, nrm, Spart, zpart, cpart, Spre, zpre, cpre, P, sl));
  }
  const float inv_log2e = 0.6931471805599453f;
  const unsigned grid = (unsigned)(BH * P);
  typedef const unsigned short* cus;
  DARK_TRY(allow_lds(k_bwd_fwd, BwdSmem::total));
  DARK_LAUNCH(KID_BWD_FWD, pb.st, k_bwd_fwd, dim3(grid), dim3(512), BwdSmem::total, (cus)Q, (cus)K, (cus)V, (cus)dOut, Ah,
              nrm, Spre, zpre, cpre, dQ, lam, gdv, dRn, dRd, TQ, p.H, p.L, P, sl, inv_log2e);
  {
    const long long n = BH * ((long long)kF * kD + kF) / 4;
    DARK_LAUNCH(KID_BWD_SUFFIX, pb.st, k_bwd_suffix, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, dRn, dRd, cpre, Rsn, Rsd, P,
                BH);
  }
  DARK_TRY(allow_lds(k_bwd_rev, BwdSmem::total));
  DARK_LAUNCH(KID_BWD_REV, pb.st, k_bwd_rev, dim3(grid), dim3(512), BwdSmem::total, (cus)Q, (cus)K, (cus)V, (cus)dOut, Ah, Mh,
              nrm, cpre, lam, gdv, Rsn, Rsd, dK, dV, TQ, TK, RM, p.H, p.L, P, sl, inv_log2e);
  if (dM != nullptr || dW != nullptr) {
    const long long n = (long long)p.H * ((long long)kF * kD + kD * kD) / 4;
    DARK_LAUNCH(KID_BWD_DM, pb.st, k_bwd_sum, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, TK, RM, Tsum, Rmsum, p.B, p.H,
                P);
    if (dM != nullptr)
      DARK_LAUNCH(KID_BWD_DM, pb.st, k_bwd_dm, dim3((unsigned)(p.H * (kD / 4))), dim3(256), 0, Tsum, Rmsum, M, W, dM, p.H,
                  p.w_shared, std::sqrt(pb.scale));
    if (dW != nullptr) DARK_TRY(launch_dw(pb, Tsum, 1, M, dW));  // Tsum is already summed over the batch
  }
  return DARK_OK;
}

}  // namespace dark

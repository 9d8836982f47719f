// Fused MFMA causal forward of the DARK attention library (gfx950): bf16 inputs, fp32 accumulation.
//
// out_i = sum_{l<=i} (phi(q_i) . phi(k_l)) v_l / sum_{l<=i} phi(q_i) . phi(k_l)  with the feature map
// of Section 4.1 (omega~_j = M^T w_j, Appendix B) and the factorisation of Section 2 ("Efficient
// attention via random feature kernels") applied to prefixes: the sum over l splits into the keys
// before the query's tile, which enter through the running state [S|z] = phi(K)^T [V|1], and the
// keys of the tile itself, which enter through the masked 32 x 32 block of estimated kernel values.
//
// The sequence of every (b,h) is cut into P slices so that the chip is filled:
//   k_kv_reduce (fused.hip)   state of every slice, per-feature shifts
//   k_key_norms               n'(k_l) = |M' k_l|^2 for every key (log2 domain)
//   k_kv_prefix               exclusive prefix of the slice states, brought to one running scalar
//                             shift c*_p = max of the shifts of slices 0..p
//   k_causal_scan             per (b,h, slice, 64 value columns): starts from the prefix state and
//                             walks the slice in tiles of 32 tokens
// Everything is in the log2 domain with the fp16 operands A', M' of the bidirectional path.
#include <cmath>
#include <cstdlib>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

constexpr int kCT = 32;    // tokens per tile of the scan
constexpr int kDVH = 64;   // value columns per workgroup of the scan
constexpr int kMaxP = 64;  // slices per (b,h) at most

// ---------------------------------------------------------------------------
// k_key_norms: nrm[bh][l] = |M' k_l|^2.  Workgroup = 4 waves x 64 tokens; x~^T[r][tok] = M' X^T by
// MFMA with the tokens as columns, so a token's sum of squares is a sum over registers.
// ---------------------------------------------------------------------------
template <int D, int R>
__global__ __launch_bounds__(256) void k_key_norms(const unsigned short* __restrict__ Kg,
                                                   const _Float16* __restrict__ Mh, float* __restrict__ nrm, int H,
                                                   int L, int chunks_per_bh) {
  constexpr int AS = D + 8;
  __shared__ __attribute__((aligned(16))) _Float16 Ms[R * AS];
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int bh = blockIdx.x / chunks_per_bh, chunk = blockIdx.x % chunks_per_bh;
  const int h = bh % H;
  for (int ci = tid; ci < R * D / 8; ci += 256) {
    const int row = ci / (D / 8), kc = ci % (D / 8);
    *reinterpret_cast<u32x4*>(Ms + row * AS + 8 * kc) =
        *reinterpret_cast<const u32x4*>(Mh + ((size_t)h * R + row) * D + 8 * kc);
  }
  const int t0 = chunk * 256 + 64 * wv;
  const unsigned short* Xb = Kg + (size_t)bh * L * D;
  half8 xf[2][D / 16];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = min(t0 + 32 * tt + l32, L - 1);
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      u32x4 cv = bf16x8_to_f16x8(*reinterpret_cast<const u32x4*>(Xb + (size_t)tok * D + 16 * s + 8 * hf));
      xf[tt][s] = *reinterpret_cast<half8*>(&cv);
    }
  }
  __syncthreads();
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float n2[2] = {0.f, 0.f};
#pragma unroll
  for (int rt = 0; rt < R / 32; ++rt) {
    f32x16 xt[2] = {zero16, zero16};
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      half8 a = *reinterpret_cast<const half8*>(Ms + (32 * rt + l32) * AS + 16 * s + 8 * hf);
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) xt[tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xf[tt][s], xt[tt], 0, 0, 0);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v) n2[tt] = fmaf(xt[tt][v], xt[tt][v], n2[tt]);
  }
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    n2[tt] += __shfl_xor(n2[tt], 32, 64);
    const int tok = t0 + 32 * tt + l32;
    if (hf == 0 && tok < L) nrm[(size_t)bh * L + tok] = n2[tt];
  }
}

// ---------------------------------------------------------------------------
// k_kv_prefix: per (b,h): c*_p = max over slices 0..p and all features of the per-feature shifts;
// Spre_p = sum_{p' < p} 2^(c_p'j - c*_p) S_p'j (p' ascending: the order of summation is fixed),
// same for z.  Slice p's own keys are featurised with c*_p by the scan, so nothing it adds to the
// state can exceed what k_kv_reduce already bounded.
// Workgroup = (b,h, 8 features); a thread owns 8 DV / 256 adjacent state entries.
// ---------------------------------------------------------------------------
template <int DV>
__global__ __launch_bounds__(256) void k_kv_prefix(const float* __restrict__ Spart, const float* __restrict__ zpart,
                                                   const float* __restrict__ cpart, float* __restrict__ Spre,
                                                   float* __restrict__ zpre, float* __restrict__ cpre, int m, int P) {
  constexpr int EPT = 8 * DV / 256;  // 2 or 4
  typedef float fvec __attribute__((ext_vector_type(EPT)));
  __shared__ float cmax[kMaxP];
  __shared__ float cst[kMaxP];
  const int nblk = m / 8;
  const int bh = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  // the state entries of all slices are requested before anything waits
  constexpr int PB = 16;
  const int feat = 8 * blk + (tid * EPT) / DV;
  const int col = (tid * EPT) % DV;
  fvec acc;
#pragma unroll
  for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
  float zacc = 0.f;
  for (int p0 = 0; p0 < P; p0 += PB) {
    fvec v[PB];
    float cj[PB], zv[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int p = min(p0 + u, P - 1);
      const size_t row = ((size_t)bh * P + p) * m + feat;
      v[u] = *reinterpret_cast<const fvec*>(Spart + row * DV + col);
      cj[u] = cpart[row];
      zv[u] = zpart[row];
    }
    if (p0 == 0) {
      for (int p = wv; p < P; p += 4) {
        float c = -INFINITY;
        for (int i = lane; i < m; i += 64) c = fmaxf(c, cpart[((size_t)bh * P + p) * m + i]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) c = fmaxf(c, __shfl_xor(c, o, 64));
        if (lane == 0) cmax[p] = c;
      }
      __syncthreads();
      if (tid == 0) {
        float run = -INFINITY;
        for (int p = 0; p < P; ++p) {
          run = fmaxf(run, cmax[p]);
          cst[p] = run;
        }
      }
      __syncthreads();
      if (blk == 0 && tid < P) cpre[(size_t)bh * P + tid] = cst[tid];
    }
#pragma unroll
    for (int u = 0; u < PB; ++u) {
      const int p = p0 + u;
      if (p < P) {
        const float cs = cst[p];
        const float down = p > 0 ? fast_exp2(cst[p - 1] - cs) : 0.f;
        const float f = fast_exp2(cj[u] - cs);
        const size_t row = ((size_t)bh * P + p) * m + feat;
#pragma unroll
        for (int e = 0; e < EPT; ++e) acc[e] *= down;
        zacc *= down;
        *reinterpret_cast<fvec*>(Spre + row * DV + col) = acc;
        if (col == 0) zpre[row] = zacc;
#pragma unroll
        for (int e = 0; e < EPT; ++e) acc[e] = fmaf(f, v[u][e], acc[e]);
        zacc = fmaf(f, zv[u], zacc);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// k_slice_state: [S|z] = phi_K^T [V|1] over one slice of one (b,h), all dv columns.
// Workgroup = 8 waves: wave (fg, hv) = (w % 4, w / 4) projects the 32 features 64 fg + 32 hv + [0,32)
// of each 32-token tile (tokens as MFMA columns), exponentiates, and leaves the packed features in
// an LDS patch shared with its partner (fg, 1 - hv); after the tile's barrier both waves read the
// patch with transposing loads and add phi_K^T V for all 64 features of the group to their own
// half of the value columns.  z comes from an MFMA against ones in the hv = 0 waves.
// Shifts: one per wave (32 features), set from the first tile, raised only when a logit exceeds
// it by more than kRaise; a raise is published with the features so that both waves rescale the
// rows concerned.  K tiles are double-buffered, V tiles triple-buffered (they are still being
// read after the barrier), one barrier per tile.
// ---------------------------------------------------------------------------
template <int D>
struct SsSmem {
  static constexpr int AS = D + 8;
  static constexpr size_t a_bytes = (size_t)256 * AS * 2;
  static constexpr size_t x_bytes = (size_t)kCT * AS * 2;
  static constexpr size_t v_bytes = (size_t)kCT * D * 2;
  static constexpr int TBS = 64 * 2 + 8;
  static constexpr size_t tb_bytes = (size_t)kCT * TBS;  // per feature group
  static constexpr size_t ns_bytes = (size_t)kCT * 4;
  static constexpr size_t dl_bytes = (size_t)8 * 4;
  static constexpr size_t total = a_bytes + 2 * x_bytes + 3 * v_bytes + 2 * 4 * tb_bytes + 2 * ns_bytes + 2 * dl_bytes;
};

template <int D>
__global__ __launch_bounds__(512, 1) void k_slice_state(const unsigned short* __restrict__ Kg,
                                                        const unsigned short* __restrict__ Vg,
                                                        const _Float16* __restrict__ Ah,
                                                        const float* __restrict__ nrm, float* __restrict__ Spart,
                                                        float* __restrict__ zpart, float* __restrict__ cpart, int H,
                                                        int L, int P, int slice_len) {
  using SM = SsSmem<D>;
  constexpr int DVT = D, DVW = D / 2, NCT = DVW / 32, m = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16* Asl = reinterpret_cast<_Float16*>(smem);
  unsigned char* xb = smem + SM::a_bytes;
  unsigned char* vb = xb + 2 * SM::x_bytes;
  unsigned char* tbb = vb + 3 * SM::v_bytes;
  float* nsb = reinterpret_cast<float*>(tbb + 2 * 4 * SM::tb_bytes);
  float* dlb = nsb + 2 * kCT;

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int j16 = l32 % 16, g2 = l32 / 16;
  const int fg = wv % 4, hv = wv / 4;
  const int bh = blockIdx.x / P, p = blockIdx.x % P;
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  const int ntile = (tok_end - tok_begin + kCT - 1) / kCT;
  if (ntile <= 0) return;

  for (int ci = tid; ci < m * D / 8; ci += 512) {
    const int row = ci / (D / 8), kc = ci % (D / 8);
    *reinterpret_cast<u32x4*>(Asl + row * SM::AS + 8 * kc) =
        *reinterpret_cast<const u32x4*>(Ah + ((size_t)h * m + row) * D + 8 * kc);
  }

  constexpr int NCH = kCT * D / 8;  // 16-byte pieces of a K (or V) tile
  const bool stager = tid < NCH;
  u32x4 kreg = {0u, 0u, 0u, 0u}, vreg = {0u, 0u, 0u, 0u};
  float nreg = 0.f;
  const unsigned short* Kb = Kg + (size_t)bh * L * D;
  const unsigned short* Vb = Vg + (size_t)bh * L * DVT;
  auto load_tile = [&](int t) {
    const int t0 = tok_begin + t * kCT;
    if (stager) {
      const int tok = min(t0 + tid / (D / 8), tok_end - 1), kc = tid % (D / 8);
      kreg = *reinterpret_cast<const u32x4*>(Kb + (size_t)tok * D + 8 * kc);
      vreg = *reinterpret_cast<const u32x4*>(Vb + (size_t)tok * DVT + 8 * kc);
    }
    if (tid < kCT) {
      const int tok = t0 + tid;
      nreg = tok < tok_end ? -nrm[(size_t)bh * L + tok] : -1e30f;  // keys past the end: features exactly zero
    }
  };
  auto store_tile = [&](int t) {
    _Float16* xs = reinterpret_cast<_Float16*>(xb + (t % 2) * SM::x_bytes);
    unsigned short* vt = reinterpret_cast<unsigned short*>(vb + (t % 3) * SM::v_bytes);
    if (stager) {
      const int tok = tid / (D / 8), kc = tid % (D / 8);
      *reinterpret_cast<u32x4*>(xs + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(kreg);
      *reinterpret_cast<u32x4*>(vt + tok * DVT + 8 * (kc ^ (tok & 7))) = vreg;
    }
    if (tid < kCT) nsb[(t % 2) * kCT + tid] = nreg;
  };

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 S[2][NCT], zacc[2];
#pragma unroll
  for (int fb = 0; fb < 2; ++fb) {
    zacc[fb] = zero16;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) S[fb][ct] = zero16;
  }
  float c = 0.f;  // this wave's shift (log2 domain), wave-uniform

  load_tile(0);
  store_tile(0);
  if (ntile > 1) load_tile(1);
  __syncthreads();

  for (int t = 0; t < ntile; ++t) {
    if (t + 1 < ntile) store_tile(t + 1);
    if (t + 2 < ntile) load_tile(t + 2);
    const _Float16* xs = reinterpret_cast<const _Float16*>(xb + (t % 2) * SM::x_bytes);
    const unsigned short* vt = reinterpret_cast<const unsigned short*>(vb + (t % 3) * SM::v_bytes);
    unsigned char* tb = tbb + ((t % 2) * 4 + fg) * SM::tb_bytes;
    // --- this wave's 32 features of the tile ----------------------------------------------
    const float nk = nsb[(t % 2) * kCT + l32] - c;
    f32x16 U;
#pragma unroll
    for (int v = 0; v < 16; ++v) U[v] = nk;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const half8 a = *reinterpret_cast<const half8*>(Asl + (64 * fg + 32 * hv + l32) * SM::AS + 16 * s + 8 * hf);
      const half8 b = *reinterpret_cast<const half8*>(xs + l32 * SM::AS + 16 * s + 8 * hf);
      U = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, U, 0, 0, 0);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; v += 2) mx = max3(mx, U[v], U[v + 1]);
    float delta = 0.f;
    if (t == 0 || __any(mx > kRaise)) {  // wave-uniform; after the first tile this is rare
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      delta = mx;
      c += delta;
#pragma unroll
      for (int v = 0; v < 16; ++v) U[v] -= delta;
    }
    if (lane == 0) dlb[(t % 2) * 8 + wv] = delta;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2 w = {pack_bf16(fast_exp2(U[4 * g]), fast_exp2(U[4 * g + 1])),
                 pack_bf16(fast_exp2(U[4 * g + 2]), fast_exp2(U[4 * g + 3]))};
      *reinterpret_cast<u32x2*>(tb + l32 * SM::TBS + (32 * hv + 8 * g + 4 * hf) * 2) = w;
    }
    __syncthreads();
    // --- a raise by either wave of the pair rescales the rows of its 32 features (rare) ------
    if (t > 0) {
      const float d0 = dlb[(t % 2) * 8 + fg], d1 = dlb[(t % 2) * 8 + 4 + fg];
      if (d0 != 0.f || d1 != 0.f) {
        const float f0 = fast_exp2(-d0), f1 = fast_exp2(-d1);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          zacc[0][v] *= f0;
          zacc[1][v] *= f1;
#pragma unroll
          for (int ct = 0; ct < NCT; ++ct) {
            S[0][ct][v] *= f0;
            S[1][ct][v] *= f1;
          }
        }
      }
    }
    // --- S += phi_K^T V, z += phi_K^T 1: k-slot s of half hf is token 16 hh + 8 (s/4) + 4 hf + s%4 ---
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      u32x4 bv[NCT];
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) {
        const int tok = 16 * hh + 4 * hf + j16 / 4;
        const int chunk = (DVW * hv) / 8 + 4 * ct + 2 * g2 + (j16 % 4) / 2;
        const unsigned short* vr = vt + tok * DVT + 8 * (chunk ^ (tok & 7)) + 4 * (j16 % 2);
        u32x2 lo = lds_read_tr16(vr);
        u32x2 hi = lds_read_tr16(vr + 8 * DVT);
        bv[ct] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
#pragma unroll
      for (int fb = 0; fb < 2; ++fb) {
        const unsigned short* tr = reinterpret_cast<const unsigned short*>(tb + (16 * hh + 4 * hf + j16 / 4) * SM::TBS) +
                                   32 * fb + 16 * g2 + 4 * (j16 % 4);
        u32x2 lo = lds_read_tr16(tr);
        u32x2 hi = lds_read_tr16(tr + 8 * (SM::TBS / 2));
        u32x4 ak = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
          S[fb][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak),
                                                              *reinterpret_cast<bf16x8*>(&bv[ct]), S[fb][ct], 0, 0, 0);
        if (hv == 0) {
          u32x4 o4 = {kOnesBf16x2, kOnesBf16x2, kOnesBf16x2, kOnesBf16x2};
          zacc[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak),
                                                             *reinterpret_cast<bf16x8*>(&o4), zacc[fb], 0, 0, 0);
        }
      }
    }
  }

  // --- the slice's state ---------------------------------------------------------------------
  const size_t srow0 = ((size_t)bh * P + p) * m;
#pragma unroll
  for (int fb = 0; fb < 2; ++fb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int feat = 64 * fg + 32 * fb + 8 * (v / 4) + 4 * hf + (v % 4);
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) Spart[(srow0 + feat) * DVT + DVW * hv + 32 * ct + l32] = S[fb][ct][v];
      if (hv == 0 && l32 == 0) zpart[srow0 + feat] = zacc[fb][v];
    }
  if (hf == 0) cpart[srow0 + 64 * fg + 32 * hv + l32] = c;
}

// ---------------------------------------------------------------------------
// k_causal_scan
// Workgroup = 4 waves over one slice of one (b,h) and 64 of the value columns; wave w owns
// features [64w, 64w+64) (m = 256) and carries their rows of the state in accumulators:
// S[feat][col] as MFMA accumulators, z[feat] as the accumulators of an MFMA against ones (all 32
// columns equal, so every lane holds the z of exactly the features its phi_Q registers hold).
// Per tile of 32 tokens, with tokens as MFMA columns in both projections
// (U^T[feat][tok] = A' X^T, lane = token):
//   phi_K = exp2(U_K - n' - c*), phi_Q = exp2(U_Q - mu), mu the row maximum over the wave's features
//   P^T[k][q] = phi_K phi_Q^T over the wave's features, masked to k <= q      (intra-tile scores)
//   N[q][col] = P V  +  phi_Q S                                               (before S is updated)
//   D[q]      = row sums of P  +  phi_Q . z
//   S += phi_K^T V,  z += phi_K^T 1   (phi_K is turned through a per-wave LDS patch with
//                                      transposing reads: this contraction runs over tokens)
// Every MFMA operand that is not read from LDS is the bf16 pack of an accumulator: the 32x32
// accumulator layout (lane = column, registers = rows 8 (v/4) + 4 (lane/32) + v%4) is an operand
// layout with the contraction index permuted, and both operands of a product use the same
// permutation.  The four waves' partial (N, D, mu) meet in LDS; 256 threads combine them with the
// factors 2^(mu_w - max mu), normalise and store 16-byte pieces of whole rows.
// ---------------------------------------------------------------------------
template <int D>
struct CsSmem {
  static constexpr int AS = D + 8;                       // fp16 elements per row of A' and of an X tile
  static constexpr size_t a_bytes = (size_t)256 * AS * 2;
  static constexpr size_t x_bytes = (size_t)kCT * AS * 2;   // one tile of Q or of K
  static constexpr size_t v_bytes = (size_t)kCT * kDVH * 2;
  static constexpr int TBS = 64 * 2 + 8;                 // bytes per token row of the transpose patch
  static constexpr size_t tb_bytes = (size_t)kCT * TBS;  // per wave
  static constexpr int NBS = kDVH + 4;                   // floats per row of a partial-N tile
  static constexpr size_t nb_bytes = (size_t)kCT * NBS * 4;  // per wave
  static constexpr size_t dm_bytes = (size_t)2 * kCT * 4;    // per wave: D, mu
  static constexpr size_t ns_bytes = (size_t)kCT * 4;
  static constexpr size_t total = a_bytes + 2 * x_bytes + v_bytes + 4 * (tb_bytes + nb_bytes + dm_bytes) + ns_bytes;
};

template <int D, bool OUT_BF16>
__global__ __launch_bounds__(256, 2) void k_causal_scan(const unsigned short* __restrict__ Qg,
                                                        const unsigned short* __restrict__ Kg,
                                                        const unsigned short* __restrict__ Vg,
                                                        const _Float16* __restrict__ Ah,
                                                        const float* __restrict__ nrm,
                                                        const float* __restrict__ Spre,
                                                        const float* __restrict__ zpre,
                                                        const float* __restrict__ cpre, void* __restrict__ outp, int H,
                                                        int L, int P, int slice_len) {
  using SM = CsSmem<D>;
  constexpr int DVT = D;           // value width (dv = d)
  constexpr int NH = DVT / kDVH;   // workgroups per (b,h, slice)
  constexpr int m = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16* Asl = reinterpret_cast<_Float16*>(smem);
  _Float16* Xq = reinterpret_cast<_Float16*>(smem + SM::a_bytes);
  _Float16* Xk = reinterpret_cast<_Float16*>(smem + SM::a_bytes + SM::x_bytes);
  unsigned short* Vt = reinterpret_cast<unsigned short*>(smem + SM::a_bytes + 2 * SM::x_bytes);
  unsigned char* wbase = smem + SM::a_bytes + 2 * SM::x_bytes + SM::v_bytes;
  constexpr size_t wave_bytes = SM::tb_bytes + SM::nb_bytes + SM::dm_bytes;
  float* ns = reinterpret_cast<float*>(wbase + 4 * wave_bytes);

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  unsigned char* tb = wbase + wv * wave_bytes;
  float* nbw = reinterpret_cast<float*>(wbase + wv * wave_bytes + SM::tb_bytes);
  float* dmw = reinterpret_cast<float*>(wbase + wv * wave_bytes + SM::tb_bytes + SM::nb_bytes);

  const int half = blockIdx.x % NH;
  const int p = (blockIdx.x / NH) % P;
  const int bh = blockIdx.x / (NH * P);
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  const int ntile = (tok_end - tok_begin + kCT - 1) / kCT;
  if (ntile <= 0) return;

  // --- resident operands ---------------------------------------------------------------------
  for (int ci = tid; ci < m * D / 8; ci += 256) {
    const int row = ci / (D / 8), kc = ci % (D / 8);
    *reinterpret_cast<u32x4*>(Asl + row * SM::AS + 8 * kc) =
        *reinterpret_cast<const u32x4*>(Ah + ((size_t)h * m + row) * D + 8 * kc);
  }
  const size_t srow0 = ((size_t)bh * P + p) * m;
  const float cs = cpre[(size_t)bh * P + p];
  f32x16 S[2][2], zacc[2];
#pragma unroll
  for (int fb = 0; fb < 2; ++fb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int feat = 64 * wv + 32 * fb + 8 * (v / 4) + 4 * hf + (v % 4);
      zacc[fb][v] = zpre[srow0 + feat];
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) S[fb][ct][v] = Spre[(srow0 + feat) * DVT + half * kDVH + 32 * ct + l32];
    }

  // --- staging ---------------------------------------------------------------------------------
  constexpr int KCH = D / 64;  // 16-byte pieces of a Q (or K) tile per thread
  u32x4 qreg[KCH], kreg[KCH], vreg;
  float nreg = 0.f;
  const unsigned short* Qb = Qg + (size_t)bh * L * D;
  const unsigned short* Kb = Kg + (size_t)bh * L * D;
  const unsigned short* Vb = Vg + (size_t)bh * L * DVT + half * kDVH;
  // Rows past the end of the slice repeat its last row (in bounds, no predication); such keys get
  // the norm term -1e30, so their features are exactly zero, and such queries are never stored.
  auto load_tile = [&](int t) {
    const int t0 = tok_begin + t * kCT;
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int ci = tid + 256 * i, tok = min(t0 + ci / (D / 8), tok_end - 1), kc = ci % (D / 8);
      qreg[i] = *reinterpret_cast<const u32x4*>(Qb + (size_t)tok * D + 8 * kc);
      kreg[i] = *reinterpret_cast<const u32x4*>(Kb + (size_t)tok * D + 8 * kc);
    }
    {
      const int tok = min(t0 + tid / 8, tok_end - 1), cc = tid % 8;
      vreg = *reinterpret_cast<const u32x4*>(Vb + (size_t)tok * DVT + 8 * cc);
    }
    if (tid < kCT) {
      const int tok = t0 + tid;
      nreg = tok < tok_end ? -(nrm[(size_t)bh * L + tok] + cs) : -1e30f;
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int ci = tid + 256 * i, tok = ci / (D / 8), kc = ci % (D / 8);
      *reinterpret_cast<u32x4*>(Xq + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(qreg[i]);
      *reinterpret_cast<u32x4*>(Xk + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(kreg[i]);
    }
    {
      const int tok = tid / 8, cc = tid % 8;
      *reinterpret_cast<u32x4*>(Vt + tok * kDVH + 8 * (cc ^ (tok & 7))) = vreg;
    }
    if (tid < kCT) ns[tid] = nreg;
  };

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const u32x4 ones4 = {kOnesBf16x2, kOnesBf16x2, kOnesBf16x2, kOnesBf16x2};
  const int j16 = l32 % 16, g2 = l32 / 16;

  load_tile(0);
  store_tile();
  __syncthreads();

  for (int t = 0; t < ntile; ++t) {
    // --- projections: tokens are columns, so lane = token.  Queries first, then keys, so that
    // only one set of projection accumulators is alive at a time. ----------------------------
    u32x4 pq[2][2], pkk[2][2];  // [fb][hh]: k-slot s <-> accumulator register 8 hh + s
    float mu, den = 0.f;
    {
      f32x16 UQ[2] = {zero16, zero16};
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        const half8 bq = *reinterpret_cast<const half8*>(Xq + l32 * SM::AS + 16 * s + 8 * hf);
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
          const half8 a = *reinterpret_cast<const half8*>(Asl + (64 * wv + 32 * fb + l32) * SM::AS + 16 * s + 8 * hf);
          UQ[fb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bq, UQ[fb], 0, 0, 0);
        }
        if (s % 4 == 3) __builtin_amdgcn_sched_barrier(0);  // bounds how far operand reads run ahead
      }
      mu = -INFINITY;
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int v = 0; v < 16; v += 2) mu = max3(mu, UQ[fb][v], UQ[fb][v + 1]);
      mu = fmaxf(mu, __shfl_xor(mu, 32, 64));
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int v = 8 * hh + 2 * q;
            const float a = fast_exp2(UQ[fb][v] - mu), b = fast_exp2(UQ[fb][v + 1] - mu);
            den = fmaf(a, zacc[fb][v], den);
            den = fmaf(b, zacc[fb][v + 1], den);
            pq[fb][hh][q] = pack_bf16(a, b);
          }
    }
    {
      const float nk = ns[l32];
      f32x16 UK[2];
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int v = 0; v < 16; ++v) UK[fb][v] = nk;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        const half8 bk = *reinterpret_cast<const half8*>(Xk + l32 * SM::AS + 16 * s + 8 * hf);
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
          const half8 a = *reinterpret_cast<const half8*>(Asl + (64 * wv + 32 * fb + l32) * SM::AS + 16 * s + 8 * hf);
          UK[fb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bk, UK[fb], 0, 0, 0);
        }
        if (s % 4 == 3) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int fb = 0; fb < 2; ++fb)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int v = 8 * hh + 2 * q;
            pkk[fb][hh][q] = pack_bf16(fast_exp2(UK[fb][v]), fast_exp2(UK[fb][v + 1]));
          }
    }
    // The next tile's rows are requested here, after the projections (whose accumulators have just
    // died), and are parked in LDS at the end of this tile.
    if (t + 1 < ntile) load_tile(t + 1);
    // phi_K of this wave, row-major [tok][feat], for the transposing reads below
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w = {pkk[fb][g / 2][2 * (g % 2)], pkk[fb][g / 2][2 * (g % 2) + 1]};
        *reinterpret_cast<u32x2*>(tb + l32 * SM::TBS + (32 * fb + 8 * g + 4 * hf) * 2) = w;
      }
    // --- intra-tile scores P^T[k][q], masked to k <= q --------------------------------------
    f32x16 Pt = zero16;
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
        Pt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pkk[fb][hh]),
                                                     *reinterpret_cast<bf16x8*>(&pq[fb][hh]), Pt, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int krow = 8 * (v / 4) + 4 * hf + (v % 4);
      Pt[v] = krow <= l32 ? Pt[v] : 0.f;
    }
    // The denominator sums the same bf16-rounded kernel values that multiply V, so the intra-tile
    // part of N / D is an exact convex combination of value rows.
    u32x4 pp[2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const unsigned w = pack_bf16(Pt[8 * hh + 2 * q], Pt[8 * hh + 2 * q + 1]);
        pp[hh][q] = w;
        den += __uint_as_float(w << 16) + __uint_as_float(w & 0xffff0000u);
      }
    den += __shfl_xor(den, 32, 64);
    // --- V fragments: k-slot s of half hf is token 16 hh + 8 (s/4) + 4 hf + s%4 -------------
    u32x4 bv[2][2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const int tok = 16 * hh + 4 * hf + j16 / 4;
        const int chunk = 4 * ct + 2 * g2 + (j16 % 4) / 2;
        const unsigned short* vr = Vt + tok * kDVH + 8 * (chunk ^ (tok & 7)) + 4 * (j16 % 2);
        u32x2 lo = lds_read_tr16(vr);
        u32x2 hi = lds_read_tr16(vr + 8 * kDVH);
        bv[hh][ct] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
    // --- numerator: intra-tile term, then the state as it was before this tile --------------
    f32x16 N[2] = {zero16, zero16};
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
        N[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pp[hh]),
                                                        *reinterpret_cast<bf16x8*>(&bv[hh][ct]), N[ct], 0, 0, 0);
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          u32x4 sb;
#pragma unroll
          for (int q = 0; q < 4; ++q) sb[q] = pack_bf16(S[fb][ct][8 * hh + 2 * q], S[fb][ct][8 * hh + 2 * q + 1]);
          N[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pq[fb][hh]),
                                                          *reinterpret_cast<bf16x8*>(&sb), N[ct], 0, 0, 0);
        }
    // --- state update: contraction over the tile's tokens -----------------------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int fb = 0; fb < 2; ++fb)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const unsigned short* tr = reinterpret_cast<const unsigned short*>(tb + (16 * hh + 4 * hf + j16 / 4) * SM::TBS) +
                                   32 * fb + 16 * g2 + 4 * (j16 % 4);
        u32x2 lo = lds_read_tr16(tr);
        u32x2 hi = lds_read_tr16(tr + 8 * (SM::TBS / 2));
        u32x4 ak = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
          S[fb][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak),
                                                              *reinterpret_cast<bf16x8*>(&bv[hh][ct]), S[fb][ct], 0, 0, 0);
        u32x4 o4 = ones4;
        zacc[fb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak),
                                                           *reinterpret_cast<bf16x8*>(&o4), zacc[fb], 0, 0, 0);
      }
    // --- partial results of this wave --------------------------------------------------------
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int v = 0; v < 16; ++v) nbw[(8 * (v / 4) + 4 * hf + (v % 4)) * SM::NBS + 32 * ct + l32] = N[ct][v];
    if (hf == 0) {
      dmw[l32] = den;
      dmw[kCT + l32] = mu;
    }
    __syncthreads();
    // --- combine the four waves, normalise, store --------------------------------------------
    {
      const int q = tid / 8, dg = tid % 8;
      float muw[4], mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        muw[w] = reinterpret_cast<const float*>(wbase + w * wave_bytes + SM::tb_bytes + SM::nb_bytes)[kCT + q];
        mx = fmaxf(mx, muw[w]);
      }
      float dsum = 0.f, num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float f = fast_exp2(muw[w] - mx);
        dsum = fmaf(f, reinterpret_cast<const float*>(wbase + w * wave_bytes + SM::tb_bytes + SM::nb_bytes)[q], dsum);
        const float* np = reinterpret_cast<const float*>(wbase + w * wave_bytes + SM::tb_bytes) + q * SM::NBS + 8 * dg;
        const f32x4 a = *reinterpret_cast<const f32x4*>(np), b = *reinterpret_cast<const f32x4*>(np + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          num[e] = fmaf(f, a[e], num[e]);
          num[4 + e] = fmaf(f, b[e], num[4 + e]);
        }
      }
      const float inv = 1.0f / dsum;
      const int tok = tok_begin + t * kCT + q;
      if (tok < tok_end) {
        const size_t o = ((size_t)bh * L + tok) * DVT + half * kDVH + 8 * dg;
        if (OUT_BF16) {
          u32x4 w = {pack_bf16(num[0] * inv, num[1] * inv), pack_bf16(num[2] * inv, num[3] * inv),
                     pack_bf16(num[4] * inv, num[5] * inv), pack_bf16(num[6] * inv, num[7] * inv)};
          *reinterpret_cast<u32x4*>(reinterpret_cast<unsigned short*>(outp) + o) = w;
        } else {
          float* op = reinterpret_cast<float*>(outp) + o;
          *reinterpret_cast<f32x4*>(op) = f32x4{num[0] * inv, num[1] * inv, num[2] * inv, num[3] * inv};
          *reinterpret_cast<f32x4*>(op + 4) = f32x4{num[4] * inv, num[5] * inv, num[6] * inv, num[7] * inv};
        }
      }
    }
    if (t + 1 < ntile) store_tile();
    __syncthreads();
  }
}

int env_int(const char* name, int dflt) {
  const char* s = std::getenv(name);
  if (s == nullptr || *s == 0) return dflt;
  const int v = std::atoi(s);
  return v > 0 ? v : dflt;
}

template <int D>
dark_status launch_causal(const Problem& pb, const void* Q, const void* K, const void* V, const _Float16* Ah,
                          const _Float16* Mh, float* Spart, float* zpart, float* cpart, float* Spre, float* zpre,
                          float* cpre, float* nrm, void* out, int P, int slice_len) {
  const dark_params& p = pb.p;
  const unsigned BH = (unsigned)pb.BH();
  const int chunks_per_bh = (p.L + 255) / 256;
  DARK_LAUNCH(KID_KEY_NORMS, pb.st, (k_key_norms<D, D>), dim3(BH * chunks_per_bh), dim3(256), 0,
              (const unsigned short*)K, Mh, nrm, p.H, p.L, chunks_per_bh);
  if (env_int("DARK_CS_STATE", D == 128 ? 1 : 2) == 1) {
    auto kern = k_slice_state<D>;
    DARK_TRY(allow_lds(kern, SsSmem<D>::total));
    DARK_LAUNCH(KID_CAUSAL_STATE, pb.st, kern, dim3(BH * P), dim3(512), SsSmem<D>::total, (const unsigned short*)K,
                (const unsigned short*)V, Ah, nrm, Spart, zpart, cpart, p.H, p.L, P, slice_len);
  } else {
    DARK_TRY(fused_launch_kv_reduce(pb, K, V, Ah, Mh, Spart, zpart, cpart, P, slice_len));
  }
  DARK_LAUNCH(KID_CAUSAL_PREFIX, pb.st, (k_kv_prefix<D>), dim3(BH * (p.m / 8)), dim3(256), 0, Spart, zpart, cpart,
              Spre, zpre, cpre, p.m, P);
  const size_t lds = CsSmem<D>::total;
  const unsigned grid = BH * P * (D / kDVH);
  if (p.out_dtype == DARK_BF16) {
    auto kern = k_causal_scan<D, true>;
    DARK_TRY(allow_lds(kern, lds));
    DARK_LAUNCH(KID_CAUSAL_SCAN, pb.st, kern, dim3(grid), dim3(256), lds, (const unsigned short*)Q,
                (const unsigned short*)K, (const unsigned short*)V, Ah, nrm, Spre, zpre, cpre, out, p.H, p.L, P,
                slice_len);
  } else {
    auto kern = k_causal_scan<D, false>;
    DARK_TRY(allow_lds(kern, lds));
    DARK_LAUNCH(KID_CAUSAL_SCAN, pb.st, kern, dim3(grid), dim3(256), lds, (const unsigned short*)Q,
                (const unsigned short*)K, (const unsigned short*)V, Ah, nrm, Spre, zpre, cpre, out, p.H, p.L, P,
                slice_len);
  }
  return DARK_OK;
}

}  // namespace

bool fused_causal_supported(const Problem& pb) {
  const dark_params& p = pb.p;
  if (p.io_dtype != DARK_BF16) return false;
  const bool shape64 = p.d == 64 && p.r == 64 && p.dv == 64;
  const bool shape128 = p.d == 128 && p.r == 128 && p.dv == 128;
  return (shape64 || shape128) && p.m == 256;
}

dark_status fused_attn_causal_fwd(const Problem& pb, Arena& ar, const void* Q, const void* K, const void* V,
                                  const float* M, const float* W, void* out) {
  const dark_params& p = pb.p;
  const long long BH = pb.BH();
  // Slices: enough workgroups for every CU (one fits per CU), whole 64-token tiles of the key pass.
  const int halves = p.dv / kDVH;
  long long want = env_int("DARK_CS_WGS", 512) / (BH * halves);
  want = want < 1 ? 1 : (want > kMaxP ? kMaxP : want);
  int sl = (int)((p.L + want - 1) / want);
  sl = ((sl + kTile - 1) / kTile) * kTile;
  if (sl < kTile) sl = kTile;
  const int P = p.L > 0 ? (p.L + sl - 1) / sl : 1;

  const size_t nstate = (size_t)BH * P * p.m;
  _Float16* Ah = ar.take<_Float16>((size_t)p.H * p.m * p.d);
  _Float16* Mh = ar.take<_Float16>((size_t)p.H * p.r * p.d);
  float* Spart = ar.take<float>(nstate * p.dv);
  float* zpart = ar.take<float>(nstate);
  float* cpart = ar.take<float>(nstate);
  float* Spre = ar.take<float>(nstate * p.dv);
  float* zpre = ar.take<float>(nstate);
  float* cpre = ar.take<float>((size_t)BH * P);
  float* nrm = ar.take<float>((size_t)BH * (p.L > 0 ? p.L : 1));
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;
  if (p.L == 0 || BH == 0) return DARK_OK;

  DARK_TRY(fused_launch_prep(pb, M, W, Ah, Mh));
  if (p.d == 64)
    return launch_causal<64>(pb, Q, K, V, Ah, Mh, Spart, zpart, cpart, Spre, zpre, cpre, nrm, out, P, sl);
  return launch_causal<128>(pb, Q, K, V, Ah, Mh, Spart, zpart, cpart, Spre, zpre, cpre, nrm, out, P, sl);
}

}  // namespace dark

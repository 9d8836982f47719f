// Fused MFMA causal forward of the DARK attention library (gfx950): bf16 inputs, fp32 accumulation.
//
// out_i = sum_{l<=i} (phi(q_i) . phi(k_l)) v_l / sum_{l<=i} phi(q_i) . phi(k_l)  with the feature map
// of Section 4.1 (omega~_j = M^T w_j, Appendix B) and the factorisation of Section 2 ("Efficient
// attention via random feature kernels") applied to prefixes: the sum over l splits into the keys
// before the query's tile, which enter through the running state [S|z] = phi(K)^T [V|1], and the
// keys of the tile itself, which enter through the masked 32 x 32 block of estimated kernel values.
//
// The sequence of every (b,h) is cut into P slices so that the chip is filled:
//   k_kv_reduce (fused.hip) or k_slice_state   state of every slice, per-feature shifts
//   k_key_norms               n'(k_l) = |M' k_l|^2 for every key (log2 domain)
//   k_kv_prefix               exclusive prefix of the slice states, brought to one running scalar
//                             shift c*_p = max of the shifts of slices 0..p
//   k_causal_scan (fused_scan.hip)   per (b,h, slice): starts from the prefix state and walks the
//                             slice in tiles of 32 tokens
// (k_kv_reduce serves d = 64; the wide head uses k_slice_state, which keeps its accumulators within
// the register file.)
// Everything is in the log2 domain with the fp16 operands A', M' of the bidirectional path.
#include <cmath>
#include <cstdlib>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

constexpr int kCT = 32;    // tokens per tile of the scan
constexpr int kMaxP = 64;  // slices per (b,h) at most

// ---------------------------------------------------------------------------
// k_key_norms: nrm[bh][l] = |M' k_l|^2.  Workgroup = 4 waves x 64 tokens per chunk; x~^T[r][tok] = M' X^T by
// MFMA with the tokens as columns, so a token's sum of squares is a sum over registers.
// ---------------------------------------------------------------------------
template <int D, int R>
__global__ __launch_bounds__(256, 4) void k_key_norms(const unsigned short* __restrict__ Kg,
                                                      const _Float16* __restrict__ Mh, float* __restrict__ nrm, int H,
                                                      int L, int blocks_per_bh, int chunks_per_block) {
  constexpr int AS = D + 8;
  __shared__ __attribute__((aligned(16))) _Float16 Ms[R * AS];
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int bh = blockIdx.x / blocks_per_bh, blk = blockIdx.x % blocks_per_bh;
  const int h = bh % H;
  const unsigned short* Xb = Kg + (size_t)bh * L * D;
  for (int ci = tid; ci < R * D / 8; ci += 256) {
    const int row = ci / (D / 8), kc = ci % (D / 8);
    *reinterpret_cast<u32x4*>(Ms + row * AS + 8 * kc) =
        *reinterpret_cast<const u32x4*>(Mh + ((size_t)h * R + row) * D + 8 * kc);
  }
  __syncthreads();
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int c_begin = blk * chunks_per_block;
  const int c_end = min(c_begin + chunks_per_block, (L + 255) / 256);
  // A wave walks its 64 tokens of every 256-token chunk in blocks of 32; few registers, so that four
  // workgroups share a CU and their memory waits overlap.
  for (int chunk = c_begin; chunk < c_end; ++chunk) {
    // X fragments (B operand) of both 32-token blocks: token = tok0 + l32, k = 16 s + 8 hf + [0,8); rows
    // past the end repeat the last row and are never stored.  All loads are issued before the first is
    // converted, so the wave waits for memory once per chunk.
    constexpr int NB = D <= 64 ? 2 : 1;  // blocks fetched together (registers)
    u32x4 raw[2][D / 16];
#pragma unroll
    for (int tt = 0; tt < NB; ++tt) {
      const int tok = min(chunk * 256 + 64 * wv + 32 * tt + l32, L - 1);
#pragma unroll
      for (int s = 0; s < D / 16; ++s) raw[tt][s] = *reinterpret_cast<const u32x4*>(Xb + (size_t)tok * D + 16 * s + 8 * hf);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int tok0 = chunk * 256 + 64 * wv + 32 * tt;
      if (tok0 >= L) break;  // wave-uniform
      if (tt >= NB) {
        const int tok = min(tok0 + l32, L - 1);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) raw[tt][s] = *reinterpret_cast<const u32x4*>(Xb + (size_t)tok * D + 16 * s + 8 * hf);
      }
      half8 xf[D / 16];
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        u32x4 cv = bf16x8_to_f16x8(raw[tt][s]);
        xf[s] = *reinterpret_cast<half8*>(&cv);
      }
      float n2 = 0.f;
#pragma unroll
      for (int rt = 0; rt < R / 32; ++rt) {
        f32x16 xt = zero16;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
          half8 a = *reinterpret_cast<const half8*>(Ms + (32 * rt + l32) * AS + 16 * s + 8 * hf);
          xt = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xf[s], xt, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) n2 = fmaf(xt[v], xt[v], n2);
      }
      n2 += __shfl_xor(n2, 32, 64);
      if (hf == 0 && tok0 + l32 < L) nrm[(size_t)bh * L + tok0 + l32] = n2;
    }
  }
}

// ---------------------------------------------------------------------------
// k_kv_prefix: per (b,h): c*_p = max over slices 0..p and all features of the per-feature shifts;
// Spre_p = sum_{p' < p} 2^(c_p'j - c*_p) S_p'j (p' ascending: the order of summation is fixed),
// same for z.  Slice p's own keys are featurised with c*_p by the scan, so nothing it adds to the
// state can exceed what k_kv_reduce already bounded.
// Workgroup = (b,h, 8 features); a thread owns 8 DV / 256 adjacent state entries.
// PB: slices whose entries a thread requests together (the smallest of 4, 8, 16 that covers P, so that a short
// chain of slices does not request its last slice over and over to fill the batch).
// ---------------------------------------------------------------------------
template <int DV, int PB>
__global__ __launch_bounds__(256) void k_kv_prefix(const unsigned short* __restrict__ Spart,
                                                   const float* __restrict__ zpart,
                                                   const float* __restrict__ cpart, float* __restrict__ Spre,
                                                   float* __restrict__ zpre, float* __restrict__ cpre, int m, int P) {
  constexpr int EPT = 8 * DV / 256;  // 2 or 4
  typedef float fvec __attribute__((ext_vector_type(EPT)));
  __shared__ float cmax[kMaxP];
  __shared__ float cst[kMaxP];
  __shared__ float cl[16][256];
  const int nblk = m / 8;
  const int bh = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  // the state entries of all slices are requested before anything waits
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
      {  // EPT bf16 values of the slice state
        typedef unsigned uvec __attribute__((ext_vector_type(EPT / 2)));
        const uvec w = *reinterpret_cast<const uvec*>(Spart + row * DV + col);
#pragma unroll
        for (int e = 0; e < EPT / 2; ++e) {
          v[u][2 * e] = __uint_as_float(w[e] << 16);
          v[u][2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
      }
      cj[u] = cpart[row];
      zv[u] = zpart[row];
    }
    if (p0 == 0) {
      // largest shift of every slice: sixteen slices' shifts are fetched together (one memory round trip),
      // parked in LDS, and reduced a slice per wave
      for (int q0 = 0; q0 < P; q0 += 16) {
        for (int i0 = 0; i0 < m; i0 += 256) {
          float cv[16];
#pragma unroll
          for (int u = 0; u < 16; ++u)
            cv[u] = i0 + tid < m ? cpart[((size_t)bh * P + min(q0 + u, P - 1)) * m + i0 + tid] : -INFINITY;
          if (i0 > 0) {
#pragma unroll
            for (int u = 0; u < 16; ++u) cv[u] = fmaxf(cv[u], cl[u][tid]);
          }
#pragma unroll
          for (int u = 0; u < 16; ++u) cl[u][tid] = cv[u];
        }
        __syncthreads();
        for (int u = wv; u < 16 && q0 + u < P; u += 4) {
          float c = fmaxf(fmaxf(cl[u][lane], cl[u][lane + 64]), fmaxf(cl[u][lane + 128], cl[u][lane + 192]));
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) c = fmaxf(c, __shfl_xor(c, o, 64));
          if (lane == 0) cmax[q0 + u] = c;
        }
        __syncthreads();
      }
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
// Workgroup = 8 waves: wave w owns the 32 features 32 w + [0,32) (w = 2 fg + hv below): it projects them for
// each 32-token tile (tokens as MFMA columns), exponentiates, leaves the packed features in LDS, reads them
// back with transposing loads (its own writes: no barrier) and adds phi_K^T V for all value columns and
// phi_K^T 1 to its accumulators.  Nothing passes between waves but the tiles themselves, so the one barrier
// of a step is the one that publishes the next tiles, and the waves are free to drift apart inside a step.
// Shifts: one per wave (32 features), set from the first tile, raised only when a logit exceeds
// it by more than kRaise; a raise rescales the wave's accumulators.
// NORMS: the key norms n'(k_l) = |M' k_l|^2 are formed here as well (and written out for the scan), one
// tile ahead of their use: every wave projects the next tile onto its 16 rows of M' (16x16x32 MFMAs, the
// rows resident in registers) and leaves 32 partial sums of squares; after the tile's barrier every lane
// adds the eight partial sums of its token in a fixed order.  Otherwise the norms are read from nrm.
// K tiles are stored two tiles ahead (three buffers: the tile being featurised, the one whose norms are
// being formed, the one being written), V tiles one ahead, at the end of a step.
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
  static constexpr size_t np_bytes = (size_t)kCT * 8 * 4;  // partial norms of a tile: [tok][wave]
  static constexpr size_t total =
      a_bytes + 3 * x_bytes + 3 * v_bytes + 2 * 4 * tb_bytes + 3 * ns_bytes + 2 * dl_bytes + 2 * np_bytes;
};

template <int D, bool NORMS>
__global__ __launch_bounds__(512, 1) void k_slice_state(const unsigned short* __restrict__ Kg,
                                                        const unsigned short* __restrict__ Vg,
                                                        const _Float16* __restrict__ Ah,
                                                        const _Float16* __restrict__ Mh, float* __restrict__ nrm,
                                                        unsigned short* __restrict__ Spart,
                                                        float* __restrict__ zpart, float* __restrict__ cpart, int H,
                                                        int L, int P, int slice_len) {
  using SM = SsSmem<D>;
  constexpr int DVT = D, NCT = D / 32, m = 256;
  static_assert(!NORMS || D == 128, "the norm stage gives every wave 16 rows of M': r = d = 128");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16* Asl = reinterpret_cast<_Float16*>(smem);
  unsigned char* xb = smem + SM::a_bytes;
  unsigned char* vb = xb + 3 * SM::x_bytes;
  unsigned char* tbb = vb + 3 * SM::v_bytes;
  float* nsb = reinterpret_cast<float*>(tbb + 2 * 4 * SM::tb_bytes);
  float* dlb = nsb + 3 * kCT;
  float* npb = dlb + 2 * 8;

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int j16 = l32 % 16, g2 = l32 / 16;
  const int l16 = lane % 16, g16 = lane / 16;
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
  // norm stage: rows 16 wv + [0,16) of M' as the A operand of 16x16x32 MFMAs (lane = row l16, k = 32 s + 8 g16 + [0,8))
  half8 mf[NORMS ? D / 32 : 1];
  if (NORMS) {
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
      mf[s] = *reinterpret_cast<const half8*>(Mh + ((size_t)h * D + 16 * wv + l16) * D + 32 * s + 8 * g16);
  }

  constexpr int NCH = kCT * D / 8;  // 16-byte pieces of a K (or V) tile
  const bool stager = tid < NCH;
  // rows in flight from global memory, by tile parity: K four tiles ahead of its use (two ahead of its store),
  // V three (two); a request is two steps old when its store needs it, which covers the latency under load
  u32x4 kregs[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}}, vregs[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
  float nregs[2] = {0.f, 0.f};
  const unsigned short* Kb = Kg + (size_t)bh * L * D;
  const unsigned short* Vb = Vg + (size_t)bh * L * DVT;
  auto load_k = [&](int t, u32x4& kreg, float& nreg) {
    const int t0 = tok_begin + t * kCT;
    if (stager) {
      const int tok = min(t0 + tid / (D / 8), tok_end - 1), kc = tid % (D / 8);
      kreg = *reinterpret_cast<const u32x4*>(Kb + (size_t)tok * D + 8 * kc);
    }
    // no arithmetic on the loaded value here: it would make the wave wait for everything above
    if (!NORMS) nreg = nrm[(size_t)bh * L + min(t0 + tid % kCT, tok_end - 1)];
  };
  auto load_v = [&](int t, u32x4& vreg) {
    const int t0 = tok_begin + t * kCT;
    if (stager) {
      const int tok = min(t0 + tid / (D / 8), tok_end - 1), kc = tid % (D / 8);
      vreg = *reinterpret_cast<const u32x4*>(Vb + (size_t)tok * DVT + 8 * kc);
    }
  };
  auto store_k = [&](int t, const u32x4& kreg, const float& nreg) {
    _Float16* xs = reinterpret_cast<_Float16*>(xb + (t % 3) * SM::x_bytes);
    if (stager) {
      const int tok = tid / (D / 8), kc = tid % (D / 8);
      *reinterpret_cast<u32x4*>(xs + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(kreg);
    }
    if (!NORMS) {
      // keys past the end of the slice: features exactly zero
      const float nsv = tok_begin + t * kCT + tid % kCT < tok_end ? -nreg : -1e30f;
      if (tid < kCT) nsb[(t % 3) * kCT + tid] = nsv;
    }
  };
  auto store_v = [&](int t, const u32x4& vreg) {
    unsigned short* vt = reinterpret_cast<unsigned short*>(vb + (t % 3) * SM::v_bytes);
    if (stager) {
      const int tok = tid / (D / 8), kc = tid % (D / 8);
      *reinterpret_cast<u32x4*>(vt + tok * DVT + 8 * (kc ^ v_swz<2 * DVT>(tok))) = vreg;
    }
  };
  // this wave's partial norms of tile t (its 16 rows of M'), from the tile in LDS
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  auto partial_norms = [&](int t) {
    const _Float16* xs = reinterpret_cast<const _Float16*>(xb + (t % 3) * SM::x_bytes);
    float* np = npb + (t % 2) * kCT * 8;
    half8 xf[2][NORMS ? D / 32 : 1];
#pragma unroll
    for (int tb2 = 0; tb2 < 2; ++tb2)
#pragma unroll
      for (int s = 0; s < (NORMS ? D / 32 : 1); ++s)
        xf[tb2][s] = *reinterpret_cast<const half8*>(xs + (16 * tb2 + l16) * SM::AS + 32 * s + 8 * g16);
#pragma unroll
    for (int tb2 = 0; tb2 < 2; ++tb2) {
      f32x4 acc = zero4;  // x~[row 16 wv + 4 g16 + i][token 16 tb2 + l16]
#pragma unroll
      for (int s = 0; s < (NORMS ? D / 32 : 1); ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(mf[s], xf[tb2][s], acc, 0, 0, 0);
      float sq = acc[0] * acc[0];
      sq = fmaf(acc[1], acc[1], sq);
      sq = fmaf(acc[2], acc[2], sq);
      sq = fmaf(acc[3], acc[3], sq);
      sq += xor16(sq);
      sq += xor32(sq);
      if (g16 == 0) np[(16 * tb2 + l16) * 8 + wv] = sq;
    }
  };

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 S[NCT], zacc = zero16;  // rows: this wave's 32 features; zacc: every column alike
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) S[ct] = zero16;
  float c = 0.f;  // this wave's shift (log2 domain), wave-uniform

  // prologue: K tiles 0 and 1 and V tile 0 in LDS, K tiles 2, 3 and V tiles 1, 2 on their way, norms of tile 0
  load_k(0, kregs[0], nregs[0]);
  if (ntile > 1) load_k(1, kregs[1], nregs[1]);
  load_v(0, vregs[0]);
  store_k(0, kregs[0], nregs[0]);
  if (ntile > 1) store_k(1, kregs[1], nregs[1]);
  store_v(0, vregs[0]);
  if (ntile > 2) load_k(2, kregs[0], nregs[0]);
  if (ntile > 3) load_k(3, kregs[1], nregs[1]);
  if (ntile > 1) load_v(1, vregs[1]);
  if (ntile > 2) load_v(2, vregs[0]);
  __syncthreads();
  if (NORMS) {
    partial_norms(0);
    __syncthreads();
  }

  // one step; kr, nr: the register set of this tile's parity (holds tile t + 2), vr: the other parity's (tile t + 1)
  auto step = [&](int t, u32x4& kr, float& nr, u32x4& vr) {
    const _Float16* xs = reinterpret_cast<const _Float16*>(xb + (t % 3) * SM::x_bytes);
    const unsigned short* vt = reinterpret_cast<const unsigned short*>(vb + (t % 3) * SM::v_bytes);
    unsigned char* tb = tbb + ((t % 2) * 4 + fg) * SM::tb_bytes;
    // --- this wave's 32 features of the tile ----------------------------------------------
    float nk;
    if (NORMS) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(npb + (t % 2) * kCT * 8 + l32 * 8);
      const f32x4 b = *reinterpret_cast<const f32x4*>(npb + (t % 2) * kCT * 8 + l32 * 8 + 4);
      const float n = ((a[0] + a[1]) + (a[2] + a[3])) + ((b[0] + b[1]) + (b[2] + b[3]));
      // keys past the end of the slice: features exactly zero
      nk = (tok_begin + t * kCT + l32 < tok_end ? -n : -1e30f) - c;
      if (wv == 0 && hf == 0 && tok_begin + t * kCT + l32 < tok_end) nrm[(size_t)bh * L + tok_begin + t * kCT + l32] = n;
    } else {
      nk = nsb[(t % 3) * kCT + l32] - c;
    }
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
    if (t == 0 || __any(mx > kRaise)) {  // wave-uniform; after the first tile this is rare
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      c += mx;
#pragma unroll
      for (int v = 0; v < 16; ++v) U[v] -= mx;
      if (t > 0) {  // what has been summed under the old shift comes down to the new one
        const float f = fast_exp2(-mx);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          zacc[v] *= f;
#pragma unroll
          for (int ct = 0; ct < NCT; ++ct) S[ct][v] *= f;
        }
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2 w = {pack_bf16(fast_exp2(U[4 * g]), fast_exp2(U[4 * g + 1])),
                 pack_bf16(fast_exp2(U[4 * g + 2]), fast_exp2(U[4 * g + 3]))};
      *reinterpret_cast<u32x2*>(tb + l32 * SM::TBS + (32 * hv + 8 * g + 4 * hf) * 2) = w;
    }
    if (NORMS && t + 1 < ntile) partial_norms(t + 1);
    // --- S += phi_K^T V, z += phi_K^T 1 for this wave's features (its own half of the patch, read back
    // transposed: LDS operations of one wave complete in order); k-slot s of half hf is token
    // 16 hh + 8 (s/4) + 4 hf + s%4 ---
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      u32x4 bv[NCT];
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct) {
        const int tok = 16 * hh + 4 * hf + j16 / 4;
        const int chunk = 4 * ct + 2 * g2 + (j16 % 4) / 2;
        const unsigned short* vr = vt + tok * DVT + 8 * (chunk ^ v_swz<2 * DVT>(tok)) + 4 * (j16 % 2);
        u32x2 lo = lds_read_tr16(vr);
        u32x2 hi = lds_read_tr16(vr + 8 * DVT);
        bv[ct] = u32x4{lo[0], lo[1], hi[0], hi[1]};
      }
      const unsigned short* tr = reinterpret_cast<const unsigned short*>(tb + (16 * hh + 4 * hf + j16 / 4) * SM::TBS) +
                                 32 * hv + 16 * g2 + 4 * (j16 % 4);
      u32x2 lo = lds_read_tr16(tr);
      u32x2 hi = lds_read_tr16(tr + 8 * (SM::TBS / 2));
      u32x4 ak = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
      for (int ct = 0; ct < NCT; ++ct)
        S[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak), *reinterpret_cast<bf16x8*>(&bv[ct]),
                                                        S[ct], 0, 0, 0);
      u32x4 o4 = {kOnesBf16x2, kOnesBf16x2, kOnesBf16x2, kOnesBf16x2};
      zacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&ak), *reinterpret_cast<bf16x8*>(&o4), zacc,
                                                     0, 0, 0);
    }
    // --- the tiles to come: K two tiles ahead, V one; then the step's only barrier ------------------
    if (t + 2 < ntile) store_k(t + 2, kr, nr);
    if (t + 1 < ntile) store_v(t + 1, vr);
    if (t + 4 < ntile) load_k(t + 4, kr, nr);
    if (t + 3 < ntile) load_v(t + 3, vr);
    __syncthreads();
  };
  for (int t = 0; t < ntile; t += 2) {
    step(t, kregs[0], nregs[0], vregs[1]);
    if (t + 1 < ntile) step(t + 1, kregs[1], nregs[1], vregs[0]);
  }

  // --- the slice's state ---------------------------------------------------------------------
  const size_t srow0 = ((size_t)bh * P + p) * m;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int feat = 64 * fg + 32 * hv + 8 * (v / 4) + 4 * hf + (v % 4);
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
      Spart[(srow0 + feat) * DVT + 32 * ct + l32] = (unsigned short)(pack_bf16(S[ct][v], 0.f) & 0xffffu);
    if (l32 == 0) zpart[srow0 + feat] = zacc[v];
  }
  if (hf == 0) cpart[srow0 + 64 * fg + 32 * hv + l32] = c;
}

// The same norms for M = I: nrm[row] = (scale log2(e) / 2) |k_row|^2, with no projection: D / 8 lanes per
// key row, 16 bytes each, squares summed in fp32, the partial sums added across the row's lanes.
template <int D>
__global__ __launch_bounds__(256) void k_key_norms_identity(const unsigned short* __restrict__ Kg,
                                                            float* __restrict__ nrm, long long rows, float f) {
  constexpr int LPR = D / 8;  // lanes per row
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long row = i / LPR;
  float s = 0.f;
  if (row < rows) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(Kg + row * D + 8 * (i % LPR));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xffff0000u);
      s = fmaf(lo, lo, fmaf(hi, hi, s));
    }
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (row < rows && i % LPR == 0) nrm[row] = f * s;
}

template <int D>
dark_status launch_key_norms(const Problem& pb, const void* K, const _Float16* Mh, float* nrm) {
  const dark_params& p = pb.p;
  const long long BH = pb.BH();
  if (pb.m_identity) {
    const long long rows = BH * p.L, threads = rows * (D / 8);
    DARK_LAUNCH(KID_KEY_NORMS, pb.st, (k_key_norms_identity<D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                (const unsigned short*)K, nrm, rows, 0.5f * kLog2e * pb.scale);
    return DARK_OK;
  }
  // about 1024 workgroups (four fit a CU), each over a run of 256-token chunks of one (b,h): M' is copied
  // to LDS once per workgroup
  const int chunks_per_bh = (p.L + 255) / 256;
  int blocks_per_bh = (int)(1024 / BH);
  blocks_per_bh = blocks_per_bh < 1 ? 1 : (blocks_per_bh > chunks_per_bh ? chunks_per_bh : blocks_per_bh);
  const int chunks_per_block = (chunks_per_bh + blocks_per_bh - 1) / blocks_per_bh;
  blocks_per_bh = (chunks_per_bh + chunks_per_block - 1) / chunks_per_block;
  DARK_LAUNCH(KID_KEY_NORMS, pb.st, (k_key_norms<D, D>), dim3((unsigned)(BH * blocks_per_bh)), dim3(256), 0,
              (const unsigned short*)K, Mh, nrm, p.H, p.L, blocks_per_bh, chunks_per_block);
  return DARK_OK;
}

// Key norms, then the state of every slice by k_slice_state.
template <int D>
dark_status launch_slice_state(const Problem& pb, const void* K, const void* V, const _Float16* Ah, const _Float16* Mh,
                               float* nrm, unsigned short* Spart, float* zpart, float* cpart, int P, int slice_len) {
  const dark_params& p = pb.p;
  // d = 128 with a geometry: the state kernel forms the norms on its way (one pass over K less); identity
  // geometry: the norms need no projection and come from their own small kernel
  constexpr bool can_fold = D == 128;
  const bool fold = can_fold && !pb.m_identity;
  if (!fold) DARK_TRY((launch_key_norms<D>(pb, K, Mh, nrm)));
  auto kern = fold ? k_slice_state<D, can_fold> : k_slice_state<D, false>;
  DARK_TRY(allow_lds(kern, SsSmem<D>::total));
  DARK_LAUNCH(KID_CAUSAL_STATE, pb.st, kern, dim3((unsigned)(pb.BH() * P)), dim3(512), SsSmem<D>::total,
              (const unsigned short*)K, (const unsigned short*)V, Ah, Mh, nrm, Spart, zpart, cpart, p.H, p.L, P, slice_len);
  return DARK_OK;
}

template <int D>
dark_status launch_causal(const Problem& pb, const void* Q, const void* K, const void* V, const _Float16* Ah,
                          const _Float16* Mh, unsigned short* Spart, float* zpart, float* cpart, float* Spre, float* zpre,
                          float* cpre, float* nrm, void* out, int P, int slice_len) {
  const dark_params& p = pb.p;
  const unsigned BH = (unsigned)pb.BH();
  if (D == 128 || p.sched_cs_state == 1) {
    DARK_TRY((launch_slice_state<D>(pb, K, V, Ah, Mh, nrm, Spart, zpart, cpart, P, slice_len)));
  } else {
    // the key pass computes the key norms on its way and leaves them in nrm
    DARK_TRY(fused_launch_kv_reduce(pb, K, V, Ah, Mh, Spart, zpart, cpart, P, slice_len, nrm));
  }
  auto prefix = P <= 4 ? k_kv_prefix<D, 4> : P <= 8 ? k_kv_prefix<D, 8> : k_kv_prefix<D, 16>;
  DARK_LAUNCH(KID_CAUSAL_PREFIX, pb.st, prefix, dim3(BH * (p.m / 8)), dim3(256), 0, Spart, zpart, cpart,
              Spre, zpre, cpre, p.m, P);
  return fused_launch_scan_ws(pb, Q, K, V, Ah, nrm, Spre, zpre, cpre, out, P, slice_len);
}

}  // namespace

dark_status fused_launch_slice_state128(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                        const _Float16* Mh, float* nrm, unsigned short* Spart, float* zpart,
                                        float* cpart, int P, int slice_len) {
  return launch_slice_state<128>(pb, K, V, Ah, Mh, nrm, Spart, zpart, cpart, P, slice_len);
}

dark_status fused_causal_states64(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                  const _Float16* Mh, float* nrm, unsigned short* Spart, float* zpart, float* cpart,
                                  float* Spre, float* zpre, float* cpre, int P, int slice_len) {
  const dark_params& p = pb.p;
  if (p.d != 64 || p.dv != 64 || P > kMaxP) return DARK_EUNSUPPORTED;
  DARK_TRY(fused_launch_kv_reduce(pb, K, V, Ah, Mh, Spart, zpart, cpart, P, slice_len, nrm));
  auto prefix = P <= 4 ? k_kv_prefix<64, 4> : P <= 8 ? k_kv_prefix<64, 8> : k_kv_prefix<64, 16>;
  DARK_LAUNCH(KID_CAUSAL_PREFIX, pb.st, prefix, dim3((unsigned)(pb.BH() * (p.m / 8))), dim3(256), 0, Spart, zpart,
              cpart, Spre, zpre, cpre, p.m, P);
  return DARK_OK;
}

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
  int P, sl;
  causal_slices(pb, &P, &sl);

  const size_t nstate = (size_t)BH * P * p.m;
  // what the backward can take over goes to the caller's hand-over buffer when there is one
  Arena sv(pb.saved, pb.saved_bytes);
  const bool handover = pb.saved_mode == 1 && ar.base != nullptr;
  const CausalKeep kp = take_causal_keep(handover ? sv : ar, pb, P);
  _Float16 *Ah = kp.Ah, *Mh = kp.Mh;
  float *Spre = kp.Spre, *zpre = kp.zpre, *cpre = kp.cpre, *nrm = kp.nrm;
  unsigned short* Spart = ar.take<unsigned short>(nstate * p.dv);
  float* zpart = ar.take<float>(nstate);
  float* cpart = ar.take<float>(nstate);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow || sv.overflow) return DARK_EWORKSPACE;
  if (p.L == 0 || BH == 0) return DARK_OK;

  DARK_TRY(fused_launch_prep(pb, M, W, Ah, Mh));
  if (p.d == 64)
    return launch_causal<64>(pb, Q, K, V, Ah, Mh, Spart, zpart, cpart, Spre, zpre, cpre, nrm, out, P, sl);
  return launch_causal<128>(pb, Q, K, V, Ah, Mh, Spart, zpart, cpart, Spre, zpre, cpre, nrm, out, P, sl);
}

size_t fused_saved_causal_bytes(const Problem& pb) {
  if (!fused_causal_supported(pb) || !fused_bwd_supported(pb, true) || pb.p.path == DARK_PATH_F32) return 0;
  int P, sl;
  causal_slices(pb, &P, &sl);
  Arena a(nullptr, 0);
  (void)take_causal_keep(a, pb, P);
  return a.off;
}

}  // namespace dark

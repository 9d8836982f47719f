// Fused MFMA feature-map kernel of the DARK attention library (gfx950): bf16 in, bf16 out.
//
// phi_j(x) = exp(w_j^T (M x') - 1/2 |M x'|^2 - c) / sqrt(m),  x' = sqrt(scale) x   (Section 4.1, the
// feature map before Eq. (3); omega~_j = M^T w_j as in Appendix B), computed in the log2 domain
// from the fp16 operands A' = alpha log2(e) W M and M' = alpha sqrt(log2(e)/2) M that the attention
// kernels use as well.  The pre-exponential logits never leave registers.
//
// Workgroup = 4 waves; each wave owns 64 tokens per work item and sweeps the features in units of
// 32 with the tokens as MFMA columns (U^T[feat][tok] = A' X^T), so a token's maximum over the
// features is a maximum over registers.  Queries: one launch (a sweep for the row maxima, a sweep
// that exponentiates and stores).  Keys: the shift is the maximum over the whole (b,h) slice, so a
// first launch leaves one partial maximum per work item and the second launch reduces those.
// The feature tile is turned through a per-wave LDS stage so that the stores are 128-byte rows.
#include <cmath>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

template <int D, int R>
struct FtSmem {
  static constexpr int AS = D + 8;
  static constexpr int stage_row = 128 + 8;              // bytes: 64 bf16 plus pad
  static constexpr size_t stage_bytes = 32 * stage_row;  // per wave: 32 tokens x 64 features
  __host__ __device__ static size_t a_bytes(int m) { return (size_t)m * AS * 2; }
  static constexpr size_t m_bytes = (size_t)R * AS * 2;
  __host__ __device__ static size_t total(int m) { return a_bytes(m) + m_bytes + 4 * stage_bytes + 64; }
};

// mode 0: queries (row shifts);  1: keys, partial maxima only;  2: keys, features with the slice shift
template <int D, int R, int MODE>
__global__ __launch_bounds__(256, 2) void k_featurize(const unsigned short* __restrict__ Xg,
                                                      const _Float16* __restrict__ Ah, const _Float16* __restrict__ Mh,
                                                      unsigned short* __restrict__ phi, float* __restrict__ stab,
                                                      float* __restrict__ pmax, int H, int L, int m, int chunks_per_bh,
                                                      int n_items, int items_per_wg) {
  using SM = FtSmem<D, R>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16* Asl = reinterpret_cast<_Float16*>(smem);
  _Float16* Ms = reinterpret_cast<_Float16*>(smem + SM::a_bytes(m));
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  unsigned char* stage = smem + SM::a_bytes(m) + SM::m_bytes + wv * SM::stage_bytes;
  float* red = reinterpret_cast<float*>(smem + SM::a_bytes(m) + SM::m_bytes + 4 * SM::stage_bytes);
  const int l32 = lane % 32, hf = lane / 32;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float half_log2_m = 0.5f * log2f((float)m);

  const int item_begin = blockIdx.x * items_per_wg;
  const int item_end = min(n_items, item_begin + items_per_wg);
  int cur_bh = -1, cur_h = -1;
  float cslice = 0.f;  // keys, mode 2: the shift of the current (b,h) slice (log2 domain)
  for (int item = item_begin; item < item_end; ++item) {
    const int bh = item / chunks_per_bh, chunk = item % chunks_per_bh;
    if (bh != cur_bh) {
      const int h = bh % H;
      if (cur_bh >= 0) __syncthreads();
      if (h != cur_h) {
        for (int ci = tid; ci < m * D / 8; ci += 256) {
          const int row = ci / (D / 8), kc = ci % (D / 8);
          *reinterpret_cast<u32x4*>(Asl + row * SM::AS + 8 * kc) =
              *reinterpret_cast<const u32x4*>(Ah + ((size_t)h * m + row) * D + 8 * kc);
        }
        for (int ci = tid; ci < R * D / 8; ci += 256) {
          const int row = ci / (D / 8), kc = ci % (D / 8);
          *reinterpret_cast<u32x4*>(Ms + row * SM::AS + 8 * kc) =
              *reinterpret_cast<const u32x4*>(Mh + ((size_t)h * R + row) * D + 8 * kc);
        }
        cur_h = h;
      }
      if (MODE == 2) {  // slice shift = maximum of the partial maxima of the first launch
        float v = -INFINITY;
        for (int i = tid; i < chunks_per_bh; i += 256) v = fmaxf(v, pmax[(size_t)bh * chunks_per_bh + i]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
        if (lane == 0) red[wv] = v;
        __syncthreads();
        cslice = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
      }
      __syncthreads();
      cur_bh = bh;
    }
    const int t0 = chunk * 256 + 64 * wv;
    const bool active = t0 < L;  // wave-uniform; inactive waves still take part in the barriers below
    float wmax = -INFINITY;
    if (active) {
      const unsigned short* Xb = Xg + (size_t)bh * L * D;
      // X fragments (B operand): token = t0 + 32 tt + l32, k = 16 s + 8 hf + [0,8)
      // (all loads are issued before the first is converted: one wait for memory, not one per load)
      half8 xf[2][D / 16];
      u32x4 raw[2][D / 16];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const int tok = min(t0 + 32 * tt + l32, L - 1);  // rows past the end repeat the last row; never stored
#pragma unroll
        for (int s = 0; s < D / 16; ++s) raw[tt][s] = *reinterpret_cast<const u32x4*>(Xb + (size_t)tok * D + 16 * s + 8 * hf);
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
          u32x4 cv = bf16x8_to_f16x8(raw[tt][s]);
          xf[tt][s] = *reinterpret_cast<half8*>(&cv);
        }
      // n'(token) = |M' x|^2: x~^T[r][tok] by MFMA, squares summed over the register rows and the halves
      float nrm[2] = {0.f, 0.f};
#pragma unroll
      for (int rt = 0; rt < R / 32; ++rt) {
        f32x16 xt[2] = {zero16, zero16};
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
          half8 a = *reinterpret_cast<const half8*>(Ms + (32 * rt + l32) * SM::AS + 16 * s + 8 * hf);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) xt[tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xf[tt][s], xt[tt], 0, 0, 0);
        }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int v = 0; v < 16; ++v) nrm[tt] = fmaf(xt[tt][v], xt[tt][v], nrm[tt]);
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) nrm[tt] += __shfl_xor(nrm[tt], 32, 64);

      auto project = [&](int g, f32x16 (&U)[2]) {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
          half8 a = *reinterpret_cast<const half8*>(Asl + (32 * g + l32) * SM::AS + 16 * s + 8 * hf);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
            U[tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, xf[tt][s], s == 0 ? zero16 : U[tt], 0, 0, 0);
        }
      };
      // shift per token (log2 domain): queries and the keys' first launch need the row maxima
      float sh[2];
      if (MODE != 2) {
        float mx[2] = {-INFINITY, -INFINITY};
        for (int g = 0; g < m / 32; ++g) {
          f32x16 U[2];
          project(g, U);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int v = 0; v < 16; v += 2) mx[tt] = max3(mx[tt], U[tt][v], U[tt][v + 1]);
        }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          mx[tt] = fmaxf(mx[tt], __shfl_xor(mx[tt], 32, 64)) - nrm[tt];  // maximum logit of the row
          sh[tt] = mx[tt];
          if (t0 + 32 * tt + l32 < L) wmax = fmaxf(wmax, mx[tt]);
        }
        if (MODE == 0 && hf == 0) {
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
            if (stab != nullptr && t0 + 32 * tt + l32 < L) stab[(size_t)bh * L + t0 + 32 * tt + l32] = sh[tt] / kLog2e;
        }
      } else {
        sh[0] = sh[1] = cslice;
      }
      if (MODE != 1) {
        // exponentiate and store, two units (64 features = one 128-byte row piece) at a time
        const int row = lane / 8, ch = lane % 8;
        for (int gp = 0; gp < m / 64; ++gp) {
          f32x16 U[2][2];
          project(2 * gp, U[0]);
          project(2 * gp + 1, U[1]);
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            const float off = -nrm[tt] - sh[tt] - half_log2_m;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                u32x2 w = {pack_bf16(fast_exp2(U[u][tt][4 * g] + off), fast_exp2(U[u][tt][4 * g + 1] + off)),
                           pack_bf16(fast_exp2(U[u][tt][4 * g + 2] + off), fast_exp2(U[u][tt][4 * g + 3] + off))};
                *reinterpret_cast<u32x2*>(stage + l32 * SM::stage_row + (32 * u + 8 * g + 4 * hf) * 2) = w;
              }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
              const int tok = t0 + 32 * tt + 8 * ps + row;
              u32x4 w = *reinterpret_cast<const u32x4*>(stage + (8 * ps + row) * SM::stage_row + 16 * ch);
              if (tok < L) *reinterpret_cast<u32x4*>(phi + ((size_t)bh * L + tok) * m + 64 * gp + 8 * ch) = w;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
          }
        }
      }
    }
    if (MODE == 1) {  // one partial maximum per work item
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, o, 64));
      __syncthreads();
      if (lane == 0) red[wv] = wmax;
      __syncthreads();
      if (tid == 0) pmax[item] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    }
    if (MODE == 2 && chunk == 0 && tid == 0 && stab != nullptr) stab[bh] = cslice / kLog2e;
  }
}

template <int D, int R>
dark_status launch_feat(const Problem& pb, const void* X, const _Float16* Ah, const _Float16* Mh, int is_query,
                        void* phi, float* stab, float* pmax) {
  const dark_params& p = pb.p;
  const int chunks_per_bh = (p.L + 255) / 256;
  const int n_items = (int)(pb.BH() * chunks_per_bh);
  const int wgs = 512;
  const int items_per_wg = (n_items + wgs - 1) / wgs;
  const unsigned grid = (unsigned)((n_items + items_per_wg - 1) / items_per_wg);
  const size_t lds = FtSmem<D, R>::total(p.m);
  const unsigned short* Xp = (const unsigned short*)X;
  unsigned short* php = (unsigned short*)phi;
  if (is_query) {
    auto kern = k_featurize<D, R, 0>;
    DARK_TRY(allow_lds(kern, lds));
    DARK_LAUNCH(KID_FEATURIZE, pb.st, kern, dim3(grid), dim3(256), lds, Xp, Ah, Mh, php, stab, pmax, p.H, p.L, p.m,
                chunks_per_bh, n_items, items_per_wg);
  } else {
    auto k1 = k_featurize<D, R, 1>;
    auto k2 = k_featurize<D, R, 2>;
    DARK_TRY(allow_lds(k1, lds));
    DARK_TRY(allow_lds(k2, lds));
    DARK_LAUNCH(KID_FEATURIZE, pb.st, k1, dim3(grid), dim3(256), lds, Xp, Ah, Mh, php, stab, pmax, p.H, p.L, p.m,
                chunks_per_bh, n_items, items_per_wg);
    DARK_LAUNCH(KID_FEATURIZE, pb.st, k2, dim3(grid), dim3(256), lds, Xp, Ah, Mh, php, stab, pmax, p.H, p.L, p.m,
                chunks_per_bh, n_items, items_per_wg);
  }
  return DARK_OK;
}

}  // namespace

bool fused_featurize_supported(const Problem& pb) {
  const dark_params& p = pb.p;
  if (p.io_dtype != DARK_BF16) return false;
  const bool shape64 = p.d == 64 && p.r == 64, shape128 = p.d == 128 && p.r == 128;
  if (!shape64 && !shape128) return false;
  if (p.m % 64 != 0) return false;
  const size_t lds = shape64 ? FtSmem<64, 64>::total(p.m) : FtSmem<128, 128>::total(p.m);
  return lds <= 160 * 1024;
}

dark_status fused_featurize(const Problem& pb, Arena& ar, const void* X, const float* M, const float* W, int is_query,
                            void* phi, float* stab) {
  const dark_params& p = pb.p;
  const int chunks_per_bh = (p.L + 255) / 256;
  _Float16* Ah = ar.take<_Float16>((size_t)p.H * p.m * p.d);
  _Float16* Mh = ar.take<_Float16>((size_t)p.H * p.r * p.d);
  float* pmax = ar.take<float>((size_t)pb.BH() * chunks_per_bh);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;
  DARK_TRY(fused_launch_prep(pb, M, W, Ah, Mh));
  if (p.d == 64) return launch_feat<64, 64>(pb, X, Ah, Mh, is_query, phi, stab, pmax);
  return launch_feat<128, 128>(pb, X, Ah, Mh, is_query, phi, stab, pmax);
}

}  // namespace dark

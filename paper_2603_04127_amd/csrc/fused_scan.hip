// Causal scan of the DARK attention library (gfx950), wave-specialised: the last kernel of the fused
// MFMA causal forward (fused_causal.hip describes the pass as a whole).
//
// out_i = (phi(q_i)^T S_i) / (phi(q_i)^T z_i),  [S_i | z_i] = sum_{l <= i} phi(k_l) [v_l^T | 1]
// (Section 2, "Efficient attention via random feature kernels", restricted to prefixes; feature map of
// Section 4.1).  A workgroup walks one slice of one (b,h) in tiles of 32 tokens, starting from the
// prefix state of the slice.  The sum over l splits into the keys before the tile (the running state)
// and the keys of the tile (the masked 32 x 32 block of estimated kernel values).
//
// The eight waves of a workgroup have two jobs, one of each per SIMD (wave w and wave w + 4 share a SIMD):
//   feature waves 0..3 = (half, side): project and exponentiate the tile's queries (side 0) or keys
//     (side 1) onto the 128 features [128 half, 128 half + 128) and leave them, packed to bf16, in LDS.
//     The query wave also owns the row shift mu and phi_Q . z_old; the key wave owns z.
//   state waves 4..7 = (half, c): own the state rows of that feature half for the value columns
//     [dv c / 2, dv (c + 1) / 2): scores, read-out  N = phi_Q S_old + P V  and update  S += phi_K^T V.
// The feature waves work one tile AHEAD of the state waves, so that on every SIMD the exponentials of
// tile t + 1 (vector pipe) run beside the matrix products of tile t (matrix pipe); the feature tiles are
// double-buffered.  The two feature halves carry their own row shifts; their partial numerators meet in
// LDS, where all 512 threads combine them with the factors 2^(mu_half - max mu), normalise and store.
// Two barriers per tile.
#include <hip/hip_runtime.h>

#include <cmath>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

constexpr int kCT = 32;  // tokens per tile

template <int D>
struct WsSmem {
  static constexpr int AS = D + 8;                           // halves per row of a Q or K tile
  static constexpr int CTW = D / 64;                         // 32-column blocks of V per state wave (dv = d)
  static constexpr size_t x_bytes = (size_t)kCT * AS * 2;    // Q tile; K tile
  static constexpr size_t v_bytes = (size_t)kCT * D * 2;     // one tile of V, all columns
  static constexpr int TBS = 64 * 2 + 8;                     // bytes per token of a patch: 64 features + pad
  static constexpr size_t tb_bytes = (size_t)kCT * TBS;      // patch: [tok][64 features] of one side
  static constexpr int NBS = D + 4;                          // floats per row of a partial numerator
  static constexpr size_t nb_bytes = (size_t)kCT * NBS * 4;  // per feature half
  static constexpr size_t off_xq = 0;
  static constexpr size_t off_xk = x_bytes;
  static constexpr size_t off_v = 2 * x_bytes;                    // two tiles
  static constexpr size_t off_patch = off_v + 2 * v_bytes;        // [parity][side][group of 64 features]
  static constexpr size_t off_nb = off_patch + 16 * tb_bytes;     // [half]
  static constexpr size_t off_dmq = off_nb + 2 * nb_bytes;        // [parity][half][phi_Q . z | mu][32]
  static constexpr size_t off_den = off_dmq + 2 * 2 * 2 * kCT * 4;  // [half][32]: denominator of the half
  static constexpr size_t off_z = off_den + 2 * kCT * 4;          // [parity][256]: z before the tile
  static constexpr size_t off_ns = off_z + 2 * 256 * 4;           // [32]: -(norm + shift) of the tile's keys
  static constexpr size_t off_raw = off_ns + kCT * 4;             // Q tile, K tile as fetched (bf16, unpadded)
  static constexpr size_t total = off_raw + 2 * v_bytes;
};

template <int D, bool OUT_BF16, bool FW>
__device__ __forceinline__ void ws_body(unsigned char* smem, const unsigned short* __restrict__ Qg,
                                        const unsigned short* __restrict__ Kg, const unsigned short* __restrict__ Vg,
                                        const _Float16* __restrict__ Ah, const float* __restrict__ nrm,
                                        const float* __restrict__ Spre, const float* __restrict__ zpre,
                                        const float* __restrict__ cpre, void* __restrict__ outp, int H, int L, int P,
                                        int slice_len) {
  using SM = WsSmem<D>;
  constexpr int DVT = D, m = 256, NS = D / 16, CTW = SM::CTW;
  _Float16* Xq = reinterpret_cast<_Float16*>(smem + SM::off_xq);
  _Float16* Xk = reinterpret_cast<_Float16*>(smem + SM::off_xk);
  unsigned short* Vt2 = reinterpret_cast<unsigned short*>(smem + SM::off_v);
  unsigned char* patch0 = smem + SM::off_patch;
  float* nb0 = reinterpret_cast<float*>(smem + SM::off_nb);
  float* dmq = reinterpret_cast<float*>(smem + SM::off_dmq);
  float* dden = reinterpret_cast<float*>(smem + SM::off_den);
  float* zb = reinterpret_cast<float*>(smem + SM::off_z);
  float* ns = reinterpret_cast<float*>(smem + SM::off_ns);
  unsigned short* rawq = reinterpret_cast<unsigned short*>(smem + SM::off_raw);
  unsigned short* rawk = rawq + kCT * D;

  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int j16 = l32 % 16, g2 = l32 / 16;
  const int half = (wv % 4) / 2;  // feature half of this wave
  const int sub = wv % 2;         // feature wave: 0 = queries, 1 = keys; state wave: group of value columns
  const int p = blockIdx.x % P;
  const int bh = blockIdx.x / P;
  const int h = bh % H;
  const int tok_begin = p * slice_len;
  const int tok_end = min(L, tok_begin + slice_len);
  const int ntile = (tok_end - tok_begin + kCT - 1) / kCT;
  if (ntile <= 0) return;

  auto patch = [&](int parity, int side, int g64) { return patch0 + ((parity * 2 + side) * 4 + g64) * SM::tb_bytes; };

  // --- resident operands --------------------------------------------------------------------------
  // feature wave: its 128 rows of A' (A operand of the projection: lane = feature)
  half8 afr[FW ? 4 : 1][FW ? NS : 1];
  // state wave: S rows [128 half + 32 fq, + 32) x columns [32 (CTW sub + ct), + 32)
  f32x16 S[FW ? 1 : 4][FW ? 1 : CTW];
  const size_t srow0 = ((size_t)bh * P + p) * m;
  const float cs = cpre[(size_t)bh * P + p];
  if (FW) {
#pragma unroll
    for (int fq = 0; fq < 4; ++fq)
#pragma unroll
      for (int s = 0; s < NS; ++s)
        afr[fq][s] = *reinterpret_cast<const half8*>(Ah + ((size_t)h * m + 128 * half + 32 * fq + l32) * D + 16 * s + 8 * hf);
  } else {
#pragma unroll
    for (int fq = 0; fq < 4; ++fq)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int feat = 128 * half + 32 * fq + 8 * (v / 4) + 4 * hf + (v % 4);
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) S[fq][ct][v] = Spre[(srow0 + feat) * DVT + 32 * (CTW * sub + ct) + l32];
      }
  }
  if (tid < 256) zb[tid] = zpre[srow0 + tid];  // z before tile 0
  float zacc[4] = {0.f, 0.f, 0.f, 0.f};       // key waves: z of the features 128 half + 32 fq + l32
  if (FW && sub == 1) {
#pragma unroll
    for (int fq = 0; fq < 4; ++fq) zacc[fq] = zpre[srow0 + 128 * half + 32 * fq + l32];
  }

  // --- staging -----------------------------------------------------------------------------------
  // Q, K and V tiles go straight to LDS (no staging registers are held while a tile is worked on); Q and K
  // are then converted bf16 -> fp16 in place of the tile the feature waves have finished with.  Every
  // thread converts the 16 bytes its own lane has fetched, so its own wait is all the ordering that needs.
  constexpr int NCH = kCT * D / 8;  // 16-byte pieces of a Q (or K) tile: 512 or 256
  float nreg = 0.f;
  const unsigned short* Qb = Qg + (size_t)bh * L * D;
  const unsigned short* Kb = Kg + (size_t)bh * L * D;
  const unsigned short* Vb = Vg + (size_t)bh * L * DVT;
  auto dma_v = [&](int t, int tid) {
    // a wave moves a 1 KB run of whole rows (64 / CPR rows of CPR 16-byte chunks); the XOR swizzle of the
    // chunks is applied on the source side
    constexpr int CPR = DVT / 8, RPW = 64 / CPR;
    if (tid / 64 < kCT / RPW) {
      const int t0 = tok_begin + t * kCT;
      const int ln = tid % 64, r = RPW * (tid / 64) + ln / CPR, pos = ln % CPR;
      const int tok = min(t0 + r, tok_end - 1), cc = pos ^ v_swz<2 * DVT>(r);
      dma16_to_lds(Vb + (size_t)tok * DVT + 8 * cc, Vt2 + (t % 2) * kCT * DVT + (tid / 64) * 512);
    }
  };
  auto dma_x = [&](int t, int tid) {
    const int t0 = tok_begin + t * kCT;
    const int ci = tid % NCH, tok = min(t0 + ci / (D / 8), tok_end - 1), kc = ci % (D / 8);
    if (NCH == 512) {
      dma16_to_lds(Qb + (size_t)tok * D + 8 * kc, rawq + (tid / 64) * 512);
      dma16_to_lds(Kb + (size_t)tok * D + 8 * kc, rawk + (tid / 64) * 512);
    } else {  // waves 0..3 fetch Q, the others K
      dma16_to_lds((tid < NCH ? Qb : Kb) + (size_t)tok * D + 8 * kc, (tid < NCH ? rawq : rawk) + ((tid % NCH) / 64) * 512);
    }
    nreg = nrm[(size_t)bh * L + min(t0 + tid % kCT, tok_end - 1)];
  };
  auto store_x = [&](int t, int tid) {  // after wait_vmcnt0()
    const int ci = tid % NCH, tok = ci / (D / 8), kc = ci % (D / 8);
    if (NCH == 512) {
      const u32x4 q = *reinterpret_cast<const u32x4*>(rawq + 8 * ci), k = *reinterpret_cast<const u32x4*>(rawk + 8 * ci);
      *reinterpret_cast<u32x4*>(Xq + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(q);
      *reinterpret_cast<u32x4*>(Xk + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(k);
    } else {
      const u32x4 q = *reinterpret_cast<const u32x4*>((tid < NCH ? rawq : rawk) + 8 * ci);
      *reinterpret_cast<u32x4*>((tid < NCH ? Xq : Xk) + tok * SM::AS + 8 * kc) = bf16x8_to_f16x8(q);
    }
    const float nsv = tok_begin + t * kCT + tid % kCT < tok_end ? -(nreg + cs) : -1e30f;
    if (tid < kCT) ns[tid] = nsv;
  };

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // A side's features as an operand fragment with the accumulator's permutation of the contraction
  // index: k-slots 0..3 <-> features 16 hh + 4 hf + [0,4) of block fb, slots 4..7 <-> those + 8.
  auto read_frag = [&](const unsigned char* pt, int fb, int hh) {
    const unsigned char* pr = pt + l32 * SM::TBS + (32 * fb + 16 * hh + 4 * hf) * 2;
    const u32x2 lo = *reinterpret_cast<const u32x2*>(pr), hi = *reinterpret_cast<const u32x2*>(pr + 16);
    return u32x4{lo[0], lo[1], hi[0], hi[1]};
  };
  // phi_K^T fragments (rows = 32 features of a patch, contraction over tokens)
  auto k_frag = [&](const unsigned char* pt, int fb, int hh) {
    const unsigned short* tr = reinterpret_cast<const unsigned short*>(pt + (16 * hh + 4 * hf + j16 / 4) * SM::TBS) +
                               32 * fb + 16 * g2 + 4 * (j16 % 4);
    const u32x2 l2 = lds_read_tr16(tr), h2 = lds_read_tr16(tr + 8 * (SM::TBS / 2));
    return u32x4{l2[0], l2[1], h2[0], h2[1]};
  };

  dma_x(0, tid);
  wait_vmcnt0();
  store_x(0, tid);
  __syncthreads();

  // Step i: the feature waves take tile i + 1, the state waves tile i, everybody combines tile i.
  for (int i = -1; i < ntile; ++i) {
    int tid_o = threadIdx.x;
    asm volatile("" : "+v"(tid_o));  // thread-derived addresses are recomputed per step, not kept
    if (i + 2 < ntile) dma_x(i + 2, tid_o);
    if (i + 1 < ntile) dma_v(i + 1, tid_o);

    if (FW) {
      const int t = i + 1;
      if (t < ntile) {
        const int par = t % 2;
        const _Float16* X = sub == 0 ? Xq : Xk;
        f32x16 U[4] = {zero16, zero16, zero16, zero16};
        {
          // the fragments are requested four k-steps ahead of the products that use them
          constexpr int PF = 4;
          half8 b[PF];
#pragma unroll
          for (int s = 0; s < PF; ++s) b[s] = *reinterpret_cast<const half8*>(X + l32 * SM::AS + 16 * s + 8 * hf);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            const half8 bs = b[s % PF];
            if (s + PF < NS) b[s % PF] = *reinterpret_cast<const half8*>(X + l32 * SM::AS + 16 * (s + PF) + 8 * hf);
#pragma unroll
            for (int fq = 0; fq < 4; ++fq) U[fq] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afr[fq][s], bs, U[fq], 0, 0, 0);
          }
        }
        if (sub == 0) {
          float mu = -INFINITY, den = 0.f;
#pragma unroll
          for (int fq = 0; fq < 4; ++fq)
#pragma unroll
            for (int v = 0; v < 16; v += 2) mu = max3(mu, U[fq][v], U[fq][v + 1]);
          mu = fmaxf(mu, xor32(mu));
          const float* zt = zb + par * 256 + 128 * half;
          // z of the features this lane's registers hold: rows 8 g + 4 hf + [0,4) of block fq, as it was
          // before this tile (fetched two groups ahead of their use).  phi_Q . z uses the bf16-rounded
          // features that enter N.
          f32x4 zq_next[2] = {*reinterpret_cast<const f32x4*>(zt + 4 * hf), *reinterpret_cast<const f32x4*>(zt + 8 + 4 * hf)};
#pragma unroll
          for (int fq = 0; fq < 4; ++fq) {
            unsigned char* pt = patch(par, 0, 2 * half + fq / 2) + l32 * SM::TBS + (32 * (fq % 2) + 4 * hf) * 2;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const f32x4 zq = zq_next[g % 2];
              if (4 * fq + g + 2 < 16) zq_next[g % 2] = *reinterpret_cast<const f32x4*>(zt + 8 * (4 * fq + g + 2) + 4 * hf);
              const unsigned w0 = pack_bf16(fast_exp2(U[fq][4 * g] - mu), fast_exp2(U[fq][4 * g + 1] - mu));
              const unsigned w1 = pack_bf16(fast_exp2(U[fq][4 * g + 2] - mu), fast_exp2(U[fq][4 * g + 3] - mu));
              den = fmaf(__uint_as_float(w0 << 16), zq[0], den);
              den = fmaf(__uint_as_float(w0 & 0xffff0000u), zq[1], den);
              den = fmaf(__uint_as_float(w1 << 16), zq[2], den);
              den = fmaf(__uint_as_float(w1 & 0xffff0000u), zq[3], den);
              *reinterpret_cast<u32x2*>(pt + 16 * g) = u32x2{w0, w1};
            }
          }
          den += xor32(den);
          if (hf == 0) {
            dmq[(par * 2 + half) * 2 * kCT + l32] = den;
            dmq[(par * 2 + half) * 2 * kCT + kCT + l32] = mu;
          }
        } else {
          const float nsl = ns[l32];  // -(norm + shift) of this lane's key
#pragma unroll
          for (int fq = 0; fq < 4; ++fq) {
            unsigned char* pt = patch(par, 1, 2 * half + fq / 2) + l32 * SM::TBS + (32 * (fq % 2) + 4 * hf) * 2;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const unsigned w0 = pack_bf16(fast_exp2(U[fq][4 * g] + nsl), fast_exp2(U[fq][4 * g + 1] + nsl));
              const unsigned w1 = pack_bf16(fast_exp2(U[fq][4 * g + 2] + nsl), fast_exp2(U[fq][4 * g + 3] + nsl));
              *reinterpret_cast<u32x2*>(pt + 16 * g) = u32x2{w0, w1};
            }
          }
          // z after this tile: column sums of the bf16 features just written (the wave reads its own
          // patches back, transposed; LDS operations of one wave complete in order).  With ones as the
          // row operand and the features as columns, every row of the product is the sum over the
          // tile's tokens: lane l32 owns feature 32 fq + l32 and keeps its z in a register.
          float* zn = zb + (1 - par) * 256 + 128 * half;
          u32x4 akz[4][2];
#pragma unroll
          for (int fq = 0; fq < 4; ++fq) {
            const unsigned char* pt = patch(par, 1, 2 * half + fq / 2);
            akz[fq][0] = k_frag(pt, fq % 2, 0);
            akz[fq][1] = k_frag(pt, fq % 2, 1);
          }
#pragma unroll
          for (int fq = 0; fq < 4; ++fq) {
            u32x4 o4 = {kOnesBf16x2, kOnesBf16x2, kOnesBf16x2, kOnesBf16x2};
            f32x16 dz = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&o4),
                                                                *reinterpret_cast<bf16x8*>(&akz[fq][0]), zero16, 0, 0, 0);
            dz = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&o4),
                                                         *reinterpret_cast<bf16x8*>(&akz[fq][1]), dz, 0, 0, 0);
            zacc[fq] += dz[0];
            if (hf == 0) zn[32 * fq + l32] = zacc[fq];
          }
        }
      }
    } else if (i >= 0) {
      const int t = i, par = t % 2;
      const unsigned short* Vt = Vt2 + par * kCT * DVT;
      // Every LDS operand is requested a stage before the products that use it; the compiler is kept
      // from sinking the requests back to their uses, where each product would wait a full LDS round trip.
      // The query fragments serve the scores and every value block: they stay in registers for the tile.
      u32x4 qf[4][2], kf[2][2];
#pragma unroll
      for (int fq = 0; fq < 4; ++fq)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          qf[fq][hh] = read_frag(patch(par, 0, 2 * half + fq / 2), fq % 2, hh);
          if (fq < 2) kf[fq][hh] = read_frag(patch(par, 1, 2 * half + fq / 2), fq % 2, hh);
        }
      // V fragments of this wave's column blocks: k-slot s of half hf is token 16 hh + 8 (s/4) + 4 hf + s%4
      u32x4 bv[CTW][2];
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int tok = 16 * hh + 4 * hf + j16 / 4;
          const int chunk = 4 * (CTW * sub + ct) + 2 * g2 + (j16 % 4) / 2;
          const unsigned short* vr = Vt + tok * DVT + 8 * (chunk ^ v_swz<2 * DVT>(tok)) + 4 * (j16 % 2);
          const u32x2 lo = lds_read_tr16(vr), hi = lds_read_tr16(vr + 8 * DVT);
          bv[ct][hh] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
      __builtin_amdgcn_sched_barrier(0);
      // intra-tile scores P^T[k][q] over the half's features
      f32x16 Pt = zero16;
#pragma unroll
      for (int fq = 0; fq < 4; ++fq) {
        u32x4 k0 = kf[fq % 2][0], k1 = kf[fq % 2][1];
        if (fq + 2 < 4) {
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) kf[fq % 2][hh] = read_frag(patch(par, 1, 2 * half + (fq + 2) / 2), (fq + 2) % 2, hh);
        }
        Pt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&k0), *reinterpret_cast<bf16x8*>(&qf[fq][0]),
                                                     Pt, 0, 0, 0);
        Pt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&k1), *reinterpret_cast<bf16x8*>(&qf[fq][1]),
                                                     Pt, 0, 0, 0);
      }
      // phi_K^T fragments (transposed reads) of the first two feature blocks, for the state update
      u32x4 ak[2][2];
#pragma unroll
      for (int fq = 0; fq < 2; ++fq)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) ak[fq][hh] = k_frag(patch(par, 1, 2 * half + fq / 2), fq % 2, hh);
      __builtin_amdgcn_sched_barrier(0);
      // masked scores (k <= q), packed; the denominator sums the same bf16-rounded kernel values that
      // multiply V, so the intra-tile part of N / D is an exact convex combination of value rows
      u32x4 pp[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int v = 8 * hh + 2 * q;
          const int krow = 8 * (v / 4) + 4 * hf + (v % 4);
          const float x0 = krow <= l32 ? Pt[v] : 0.f, x1 = krow + 1 <= l32 ? Pt[v + 1] : 0.f;
          pp[hh][q] = pack_bf16(x0, x1);
        }
      if (sub == 1) {  // (the wave that shares its SIMD with the key wave, the lighter of the two)
        // denominator of the half: phi_Q . z_old from the query wave plus the row sums of the masked scores
        // (lane = query; the two half-waves hold complementary keys)
        float rs = 0.f;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
#pragma unroll
          for (int q = 0; q < 4; ++q) rs += __uint_as_float(pp[hh][q] << 16) + __uint_as_float(pp[hh][q] & 0xffff0000u);
        rs += xor32(rs);
        if (hf == 0) dden[half * kCT + l32] = dmq[(par * 2 + half) * 2 * kCT + l32] + rs;
      }
      // numerators: the state as it was before this tile, then the intra-tile term
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct) {
        f32x16 N = zero16;
#pragma unroll
        for (int fq = 0; fq < 4; ++fq)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            u32x4 sb;
#pragma unroll
            for (int q = 0; q < 4; ++q) sb[q] = pack_bf16(S[fq][ct][8 * hh + 2 * q], S[fq][ct][8 * hh + 2 * q + 1]);
            N = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&qf[fq][hh]),
                                                        *reinterpret_cast<bf16x8*>(&sb), N, 0, 0, 0);
          }
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
          N = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&pp[hh]),
                                                      *reinterpret_cast<bf16x8*>(&bv[ct][hh]), N, 0, 0, 0);
        float* nbw = nb0 + half * (SM::nb_bytes / 4) + 32 * (CTW * sub + ct) + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) nbw[(8 * (v / 4) + 4 * hf + (v % 4)) * SM::NBS] = N[v];
      }
      // state update (after every read-out above): S += phi_K^T V, feature block by feature block, the
      // fragments of block fq + 2 requested while block fq multiplies
#pragma unroll
      for (int fq = 0; fq < 4; ++fq) {
        u32x4 a0 = ak[fq % 2][0], a1 = ak[fq % 2][1];
        if (fq + 2 < 4) {
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) ak[fq % 2][hh] = k_frag(patch(par, 1, 2 * half + (fq + 2) / 2), (fq + 2) % 2, hh);
        }
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) {
          S[fq][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&a0),
                                                              *reinterpret_cast<bf16x8*>(&bv[ct][0]), S[fq][ct], 0, 0, 0);
          S[fq][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&a1),
                                                              *reinterpret_cast<bf16x8*>(&bv[ct][1]), S[fq][ct], 0, 0, 0);
        }
      }
    }
    lds_barrier();

    // the next tiles' operands: Q, K of tile i + 2 (the feature waves are done with tile i + 1), V of tile i + 1
    wait_vmcnt0();  // the tiles fetched at the top of this step have landed; nothing younger is in flight yet
    if (i + 2 < ntile) store_x(i + 2, tid_o);
    // --- combine the two feature halves of tile i, normalise, store ---------------------------------
    if (i >= 0) {
      constexpr int CPT = DVT / 16;  // output columns per thread: 4 or 8
      const int q = tid_o / 16, cg = tid_o % 16;
      const float* dq = dmq + (i % 2) * 2 * 2 * kCT;
      const float mu0 = dq[kCT + q], mu1 = dq[2 * kCT + kCT + q];
      const float mx = fmaxf(mu0, mu1);
      const float f0 = fast_exp2(mu0 - mx), f1 = fast_exp2(mu1 - mx);
      const float dsum = fmaf(f0, dden[q], f1 * dden[kCT + q]);
      const float inv = __builtin_amdgcn_rcpf(dsum);
      const float* n0 = nb0 + q * SM::NBS + CPT * cg;
      const float* n1 = n0 + SM::nb_bytes / 4;
      const int tok = tok_begin + i * kCT + q;
#pragma unroll
      for (int e4 = 0; e4 < CPT / 4; ++e4) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(n0 + 4 * e4), b = *reinterpret_cast<const f32x4*>(n1 + 4 * e4);
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = fmaf(f0, a[e], f1 * b[e]) * inv;
        if (tok < tok_end) {
          const size_t off = ((size_t)bh * L + tok) * DVT + CPT * cg + 4 * e4;
          if (OUT_BF16) {
            *reinterpret_cast<u32x2*>(reinterpret_cast<unsigned short*>(outp) + off) =
                u32x2{pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
          } else {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(outp) + off) = o;
          }
        }
      }
    }
    lds_barrier();
  }
}

template <int D, bool OUT_BF16>
__global__ __launch_bounds__(512, 1) void k_causal_scan(const unsigned short* __restrict__ Qg,
                                                         const unsigned short* __restrict__ Kg,
                                                         const unsigned short* __restrict__ Vg,
                                                         const _Float16* __restrict__ Ah,
                                                         const float* __restrict__ nrm,
                                                         const float* __restrict__ Spre,
                                                         const float* __restrict__ zpre,
                                                         const float* __restrict__ cpre, void* __restrict__ outp, int H,
                                                         int L, int P, int slice_len) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (threadIdx.x < 256)
    ws_body<D, OUT_BF16, true>(smem, Qg, Kg, Vg, Ah, nrm, Spre, zpre, cpre, outp, H, L, P, slice_len);
  else
    ws_body<D, OUT_BF16, false>(smem, Qg, Kg, Vg, Ah, nrm, Spre, zpre, cpre, outp, H, L, P, slice_len);
}

template <int D>
dark_status launch_scan(const Problem& pb, const void* Q, const void* K, const void* V, const _Float16* Ah,
                        const float* nrm, const float* Spre, const float* zpre, const float* cpre, void* out, int P,
                        int slice_len) {
  const dark_params& p = pb.p;
  const unsigned grid = (unsigned)pb.BH() * P;
  const unsigned short *Qp = (const unsigned short*)Q, *Kp = (const unsigned short*)K, *Vp = (const unsigned short*)V;
  const size_t lds = WsSmem<D>::total;
  auto kern = p.out_dtype == DARK_BF16 ? k_causal_scan<D, true> : k_causal_scan<D, false>;
  DARK_TRY(allow_lds(kern, lds));
  DARK_LAUNCH(KID_CAUSAL_SCAN, pb.st, kern, dim3(grid), dim3(512), lds, Qp, Kp, Vp, Ah, nrm, Spre, zpre, cpre, out, p.H,
              p.L, P, slice_len);
  return DARK_OK;
}

}  // namespace

dark_status fused_launch_scan_ws(const Problem& pb, const void* Q, const void* K, const void* V, const _Float16* Ah,
                                 const float* nrm, const float* Spre, const float* zpre, const float* cpre, void* out,
                                 int P, int slice_len) {
  if (pb.p.d == 64) return launch_scan<64>(pb, Q, K, V, Ah, nrm, Spre, zpre, cpre, out, P, slice_len);
  return launch_scan<128>(pb, Q, K, V, Ah, nrm, Spre, zpre, cpre, out, P, slice_len);
}

}  // namespace dark

// fp32 path of the DARK attention library: every step is a small, general fp32
// kernel (a strided batched GEMM plus element-wise / reduction kernels), composed
// on the host.  It accepts any shape and either io dtype, and is the path used
// for fp32 problems, for shapes the fused MFMA kernels do not cover, and for the
// backward pass.  Intermediates (features, chunk states) live in the caller's
// workspace.
//
// Steps follow the paper: Section 4.1 (feature map with x~ = M x, h = exp(-|x~|^2/2)),
// Appendix B (omega~ = M^T w, hence logits = x' (W M)^T), Section 2 (K'^T V first,
// then Q' times it, then normalise).
#include <cmath>

#include "common.h"

namespace dark {
namespace {

constexpr int kWave = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

__device__ inline float load_as_f32(const float* p, long long i) { return p[i]; }
__device__ inline float load_as_f32(const __hip_bfloat16* p, long long i) {
  unsigned short b = reinterpret_cast<const unsigned short*>(p)[i];
  return __uint_as_float(((unsigned)b) << 16);
}
__device__ inline void store_from_f32(float* p, long long i, float v) { p[i] = v; }
__device__ inline void store_from_f32(__hip_bfloat16* p, long long i, float v) {
  // round to nearest even
  unsigned u = __float_as_uint(v);
  unsigned r;
  if ((u & 0x7fffffffu) > 0x7f800000u) {
    r = (u >> 16) | 0x40u;  // quiet NaN
  } else {
    r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  }
  reinterpret_cast<unsigned short*>(p)[i] = (unsigned short)r;
}

// ---------------------------------------------------------------------------
// Strided, three-level batched fp32 GEMM:  C = alpha * A B + beta * C.
// A is M x K, B is K x N, C is M x N, each with arbitrary element strides, so
// transposes are free.  The innermost batch index (b2) may shorten M, N and K
// ("ragged" chunks): effective size = clamp(lim - b2 * step, 0, size) if lim > 0.
// mask == 1 writes zeros where column > row (lower-triangular result).
// E != nullptr: C = (alpha * A B + beta * C) .* E, E laid out like C (the gradient of a logit is the
// gradient of its feature times the feature, Section 4.1's exponential).
// A second product with its own operands, strides and K may be added into the same C before it is
// stored (see the x* fields): two GEMMs that would otherwise write C and then read and rewrite it.
// ---------------------------------------------------------------------------
struct Gemm {
  const float* A;
  const float* B;
  float* C;
  int M, N, K;
  long long sAm, sAk, sBk, sBn, sCm, sCn;
  int nb0, nb1, nb2;
  long long sA0, sA1, sA2, sB0, sB1, sB2, sC0, sC1, sC2;
  float alpha, beta;
  int mask;
  const float* E;  // optional: the stored value is multiplied element-wise by E (indexed like C)
  int mlim, mstep, nlim, nstep, klim, kstep;
  int modeA, modeB;  // GL_* fetch modes, set by run_gemm
  // Optional second product accumulated into the same tile (register-blocked kernel only):
  // C = alpha (A B + xA xB) + beta C, same M, N, batch counts and limits on M and N; xA == nullptr: none.
  const float* xA;
  const float* xB;
  int xK;
  long long xsAm, xsAk, xsBk, xsBn;
  long long xsA0, xsA1, xsA2, xsB0, xsB1, xsB2;
  int xklim, xkstep;
  int xmodeA, xmodeB;
};

constexpr int GT = 64;  // C tile edge
constexpr int GK = 32;  // K step

// How one operand tile (64 x GK, element (x, k) at P[x * sx + k * sk]) is fetched: 16-byte loads
// along k or along x when that index is contiguous and everything is 16-byte aligned, else scalars.
// A 16-byte load that straddles the matrix edge is issued whole and its tail zeroed afterwards, so the
// vector modes also require that the contiguous extent, rounded up to four, fits under every other
// stride of the operand (rows padded to a multiple of four floats): the over-read then stays inside
// the row's own span.
enum { GL_SCALAR = 0, GL_VEC_K = 1, GL_VEC_X = 2 };

inline int gemm_load_mode(const float* P, long long sx, long long sk, int X, int K, long long s0, long long s1,
                          long long s2) {
  const bool al = ((reinterpret_cast<uintptr_t>(P) | (uintptr_t)(s0 * 4) | (uintptr_t)(s1 * 4) | (uintptr_t)(s2 * 4)) & 15) == 0;
  if (!al) return GL_SCALAR;
  auto fits = [&](int extent, long long other) {
    const long long up = ((long long)extent + 3) & ~3LL;
    for (long long st : {other, s0, s1, s2})
      if (st != 0 && st < up) return false;
    return true;
  };
  if (sk == 1 && (sx & 3) == 0 && fits(K, sx)) return GL_VEC_K;
  if (sx == 1 && (sk & 3) == 0 && fits(X, sk)) return GL_VEC_X;
  return GL_SCALAR;
}

// A thread's fetch of the register-blocked kernel: two groups of four consecutive floats (q[u][j])
// and how many of each lie inside the matrix (n[u]).  A group is fetched with one 16-byte load
// whenever its first element is inside (see gemm_load_mode for why that is safe) and the elements
// past the edge are zeroed before the group is used, so a fetch is a single predicated load: no
// second path whose loads would have to wait for the first to return.
// The groups stay 4-vectors from the load to the park: scalarised, the register allocator would load
// into a spare tuple and copy, which again means waiting for the load right behind its issue.
typedef float quad_t __attribute__((ext_vector_type(4)));
struct Fetch {
  quad_t q[2];
  int n[2];
};

__device__ __forceinline__ void load_quad(Fetch& f, int u, const float* p, int n) {
  quad_t x = {0.f, 0.f, 0.f, 0.f};
  if (n > 0) x = *reinterpret_cast<const quad_t*>(p);
  f.q[u] = x;
  f.n[u] = n;
}

// Scalar fetch of the general kernel: this thread's 8 elements of an operand tile (64 x GK, element
// (x, k) at P[x * sx + k * sk]) into registers, zero outside the matrix or when `on` is false.
// Consecutive threads walk the smaller stride.  Every element is one predicated load into a register
// of its own, so all of them are in flight together.
__device__ __forceinline__ void gemm_fetch(float (&r)[8], const float* P, long long sx, long long sk, int x0, int Xe, int k0,
                                  int Ke, int tid, bool on) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = tid + 256 * i;
    const int k = sk <= sx ? e % GK : e / GT;
    const int x = sk <= sx ? e / GK : e % GT;
    const int gx = x0 + x, gk = k0 + k;
    r[i] = (on && gx < Xe && gk < Ke) ? P[gx * sx + gk * sk] : 0.f;
  }
}

// Parks the fetched elements in the LDS tile T[k][x].
__device__ __forceinline__ void gemm_park(float (*T)[GT + 4], const float (&r)[8], long long sx, long long sk, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int e = tid + 256 * i;
    if (sk <= sx) T[e % GK][e / GK] = r[i];
    else T[e / GT][e % GT] = r[i];
  }
}

// One output tile of the batched problem, as seen by the whole workgroup (all fields uniform).
struct GemmTile {
  const float* A;
  const float* B;
  float* C;
  const float* E;  // null if none
  int m0, n0, Me, Ne, Ke;
  const float* xA;  // second product (null if none)
  const float* xB;
  int xKe;
};

// Field by field, so that both tiles stay in scalar registers.
__device__ __forceinline__ GemmTile pick_tile(bool second, const GemmTile& a, const GemmTile& b) {
  GemmTile o;
  o.A = second ? b.A : a.A;
  o.B = second ? b.B : a.B;
  o.C = second ? b.C : a.C;
  o.E = second ? b.E : a.E;
  o.m0 = second ? b.m0 : a.m0;
  o.n0 = second ? b.n0 : a.n0;
  o.Me = second ? b.Me : a.Me;
  o.Ne = second ? b.Ne : a.Ne;
  o.Ke = second ? b.Ke : a.Ke;
  o.xA = second ? b.xA : a.xA;
  o.xB = second ? b.xB : a.xB;
  o.xKe = second ? b.xKe : a.xKe;
  return o;
}

// Tile t -> its operands and effective sizes; false if the tile lies outside the (ragged) problem.
__device__ __forceinline__ bool gemm_tile(const Gemm& g, int t, int tilesM, int tilesN, int tile_m, int tile_n, GemmTile& o) {
  const int tn = t % tilesN;
  t /= tilesN;
  const int tm = t % tilesM;
  t /= tilesM;
  const int b2 = t % g.nb2;
  t /= g.nb2;
  const int b1 = t % g.nb1;
  const int b0 = t / g.nb1;
  o.Me = g.M;
  o.Ne = g.N;
  o.Ke = g.K;
  if (g.mlim > 0) o.Me = max(0, min(g.M, g.mlim - b2 * g.mstep));
  if (g.nlim > 0) o.Ne = max(0, min(g.N, g.nlim - b2 * g.nstep));
  if (g.klim > 0) o.Ke = max(0, min(g.K, g.klim - b2 * g.kstep));
  o.m0 = tm * tile_m;
  o.n0 = tn * tile_n;
  o.A = g.A + b0 * g.sA0 + b1 * g.sA1 + b2 * g.sA2;
  o.B = g.B + b0 * g.sB0 + b1 * g.sB1 + b2 * g.sB2;
  o.C = g.C + b0 * g.sC0 + b1 * g.sC1 + b2 * g.sC2;
  o.E = g.E != nullptr ? g.E + b0 * g.sC0 + b1 * g.sC1 + b2 * g.sC2 : nullptr;
  o.xA = nullptr;
  o.xB = nullptr;
  o.xKe = 0;
  if (g.xA != nullptr) {
    o.xA = g.xA + b0 * g.xsA0 + b1 * g.xsA1 + b2 * g.xsA2;
    o.xB = g.xB + b0 * g.xsB0 + b1 * g.xsB1 + b2 * g.xsB2;
    o.xKe = g.xK;
    if (g.xklim > 0) o.xKe = max(0, min(g.xK, g.xklim - b2 * g.xkstep));
  }
  return o.m0 < o.Me && o.n0 < o.Ne;
}

// Epilogue of one 32 x 32 accumulator block whose corner is (bm0, bn0): this lane holds column
// bn0 + l32, rows bm0 + 4 hf + 8 (v / 4) + v % 4.  The old values of C (beta != 0) are fetched first,
// all in flight together, then everything is stored; the offset is laundered in between so that the
// sixteen addresses are recomputed rather than kept in registers.  A block that lies wholly inside
// the matrix takes a path without per-element branches: behind a branch the compiler can no longer
// count the stores in flight and would wait for each one to finish.  Clears the accumulator.
typedef float gemm_acc_t __attribute__((ext_vector_type(16)));
template <bool kFull, bool kBeta, bool kMul>
__device__ __forceinline__ void gemm_store_block_as(const Gemm& g, float* C, const float* E, int m_first, int Me, int gn,
                                                    int Ne, gemm_acc_t& acc) {
  long long off = m_first * g.sCm + gn * g.sCn;
  const float* cb = C + off;
  const float* eb = E + off;
  const bool col = gn < Ne;
  float cv[16], ev[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int r = 8 * (v / 4) + (v % 4);
    const bool in = kFull || (col && m_first + r < Me);
    cv[v] = kBeta ? (in ? cb[r * g.sCm] : 0.f) : 0.f;
    ev[v] = kMul ? (in ? eb[r * g.sCm] : 0.f) : 1.f;
  }
  asm volatile("" : "+v"(off));
  float* cs = C + off;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int r = 8 * (v / 4) + (v % 4);
    if (kFull || (col && m_first + r < Me)) {
      float x = g.alpha * acc[v];
      if (kBeta) x += g.beta * cv[v];
      if (kMul) x *= ev[v];
      if (g.mask == 1 && gn > m_first + r) x = 0.f;
      cs[r * g.sCm] = x;
    }
    acc[v] = 0.f;
  }
}

__device__ __forceinline__ void gemm_store_block(const Gemm& g, float* C, const float* E, int bm0, int hf, int Me, int bn0,
                                                 int l32, int Ne, gemm_acc_t& acc) {
  const bool full = bm0 + 32 <= Me && bn0 + 32 <= Ne;
  const int m_first = bm0 + 4 * hf, gn = bn0 + l32;
  if (E != nullptr && g.beta != 0.f) {
    if (full) gemm_store_block_as<true, true, true>(g, C, E, m_first, Me, gn, Ne, acc);
    else gemm_store_block_as<false, true, true>(g, C, E, m_first, Me, gn, Ne, acc);
  } else if (E != nullptr) {
    if (full) gemm_store_block_as<true, false, true>(g, C, E, m_first, Me, gn, Ne, acc);
    else gemm_store_block_as<false, false, true>(g, C, E, m_first, Me, gn, Ne, acc);
  } else if (g.beta != 0.f) {
    if (full) gemm_store_block_as<true, true, false>(g, C, E, m_first, Me, gn, Ne, acc);
    else gemm_store_block_as<false, true, false>(g, C, E, m_first, Me, gn, Ne, acc);
  } else {
    if (full) gemm_store_block_as<true, false, false>(g, C, E, m_first, Me, gn, Ne, acc);
    else gemm_store_block_as<false, false, false>(g, C, E, m_first, Me, gn, Ne, acc);
  }
}

// Persistent workgroups: each walks the output tiles blockIdx.x, blockIdx.x + gridDim.x, ... and treats
// their K steps as one stream: while step s is multiplied out of one LDS buffer, the elements of step
// s + 1 (of the same tile, or the first step of the next tile) are on their way into registers, and
// they are parked in the other buffer, so there is one barrier per step and a tile's stores overlap the
// next tile's loads.
__global__ __launch_bounds__(256, 3) void k_gemm(Gemm g, int total_tiles) {
  __shared__ __attribute__((aligned(16))) float As[2][GK][GT + 4];
  __shared__ __attribute__((aligned(16))) float Bs[2][GK][GT + 4];
  const int tilesN = (g.N + GT - 1) / GT;
  const int tilesM = (g.M + GT - 1) / GT;

  const int tid = threadIdx.x;
  // Wave w owns the 32 x 32 block (w / 2, w % 2) of the tile and accumulates it with fp32 MFMAs
  // (32x32x2: lane = (row or column, k mod 2)); the accumulator holds column lane % 32, rows
  // 8 (v / 4) + 4 (lane / 32) + v % 4.
  typedef float f32x16 __attribute__((ext_vector_type(16)));
  const int lane = tid % 64, wv = tid / 64, l32 = lane % 32, hf = lane / 32;
  const int wm = wv / 2, wn = wv % 2;

  GemmTile cur, nxt;
  int t = blockIdx.x;
  while (t < total_tiles && !gemm_tile(g, t, tilesM, tilesN, GT, GT, cur)) t += gridDim.x;
  if (t >= total_tiles) return;
  nxt = cur;
  // Every tile has at least one step (an empty contraction fetches zeros), so the stream is uniform.
  float ra[8], rb[8];
  gemm_fetch(ra, cur.A, g.sAm, g.sAk, cur.m0, cur.Me, 0, cur.Ke, tid, true);
  gemm_fetch(rb, cur.B, g.sBn, g.sBk, cur.n0, cur.Ne, 0, cur.Ke, tid, true);
  int buf = 0, k0 = 0;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  while (true) {
    gemm_park(As[buf], ra, g.sAm, g.sAk, tid);
    gemm_park(Bs[buf], rb, g.sBn, g.sBk, tid);
    // what to fetch while this step is multiplied: the tile's next step, or the next tile's first
    const bool last = k0 + GK >= cur.Ke;
    int tn = t;
    bool more = true;
    if (last) {
      tn = t + gridDim.x;
      while (tn < total_tiles && !gemm_tile(g, tn, tilesM, tilesN, GT, GT, nxt)) tn += gridDim.x;
      more = tn < total_tiles;
    }
    {
      const GemmTile f = pick_tile(last, cur, nxt);
      const int fk = last ? 0 : k0 + GK;
      gemm_fetch(ra, f.A, g.sAm, g.sAk, f.m0, f.Me, fk, f.Ke, tid, more);
      gemm_fetch(rb, f.B, g.sBn, g.sBk, f.n0, f.Ne, fk, f.Ke, tid, more);
    }
    __syncthreads();
    // a wave whose 32 x 32 block lies outside the matrix (the 65th column of [V|1] opens a tile of its own)
    // leaves the matrix pipe to the other workgroups of the CU
    if (cur.m0 + 32 * wm < cur.Me && cur.n0 + 32 * wn < cur.Ne) {
#pragma unroll
      for (int kk = 0; kk < GK; kk += 2)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[buf][kk + hf][32 * wm + l32], Bs[buf][kk + hf][32 * wn + l32], acc, 0, 0, 0);
    }
    buf ^= 1;
    if (!last) {
      k0 += GK;
      continue;
    }
    gemm_store_block(g, cur.C, cur.E, cur.m0 + 32 * wm, hf, cur.Me, cur.n0 + 32 * wn, l32, cur.Ne, acc);
    if (!more) break;
    cur = nxt;
    t = tn;
    k0 = 0;
  }
}

// ---------------------------------------------------------------------------
// Register-blocked variant of the same GEMM for operands that 16-byte loads can fetch (both in a
// GL_VEC_* mode).  The workgroup's four waves form a WM x WN grid; each wave accumulates BM x BN blocks
// of 32 x 32, so one operand fragment read from LDS feeds BN (or BM) MFMAs and a fetched element is
// reused over a tile of (32 BM WM) x (32 BN WN) instead of 64 x 64.
// ---------------------------------------------------------------------------
constexpr int RK = 16;  // K step

// LDS image of the K step of an operand tile with TX rows (A) or columns (B): element (x, k),
// k = 8 g + hf + 2 s, sits at v[g][hf][rb_row(x)][s].  A lane of half hf feeds k = hf, hf + 2, hf + 4,
// hf + 6 of a group of eight to four consecutive 32x32x2 MFMAs, and finds them in one 16-byte read.
// rb_row rotates the rows of every group of eight by the group's number: the MFMA reads (32
// consecutive x) still cover eight different 16-byte bank groups per eight lanes, and so do the
// stores of a thread that fetched along x and therefore holds x = 4 q + j (stride four rows).
template <int TX>
struct RbTile {
  float v[RK / 8][2][TX + 2][4];
};
__device__ __forceinline__ int rb_row(int x) { return (x & ~7) | ((x + ((x >> 3) & 3)) & 7); }

// How the threads split an operand tile's K step (TX x RK elements, two groups of four per thread).
// along_x (x contiguous): a thread takes four neighbouring x at NS values of s of one (g, hf);
// else (k contiguous): a thread takes the eight k of one group g for one x.
template <int TX>
struct RbSplit {
  static constexpr int combos = (TX / 4) * (RK / 8) * 2;
  static constexpr int split = 256 / combos >= 4 ? 4 : (256 / combos >= 2 ? 2 : 1);
  static constexpr int NS = 4 / split;
  static constexpr int items = TX * (RK / 8);
  static_assert(NS <= 2 && items <= 256, "a thread holds at most eight elements");
};

// What a thread fetches of every K step of an operand, fixed for the whole launch: for each of its two
// groups the position along the contiguous index (c) and along the strided one (s), relative to the
// first element of the tile's K step, the element offset from there, and whether the group exists.
struct RbLane {
  long long off[2];
  int c[2], s[2];
  bool act[2];
};

template <int TX>
__device__ __forceinline__ RbLane rb_lane(bool along_x, long long sx, long long sk, int tid) {
  typedef RbSplit<TX> S;
  const int cb = tid % S::combos, sh = tid / S::combos;
  const int xq = cb % (TX / 4), ghf = cb / (TX / 4);
  const int gq = tid % (RK / 8), xk = tid / (RK / 8);
  RbLane L;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    L.c[u] = along_x ? 4 * xq : 8 * gq + 4 * u;
    L.s[u] = along_x ? 8 * (ghf / 2) + (ghf % 2) + 2 * (S::NS * sh + u) : xk;
    L.act[u] = along_x ? (sh < S::split && u < S::NS) : tid < S::items;
    L.off[u] = L.s[u] * (along_x ? sk : sx) + L.c[u];
  }
  return L;
}

// This thread's share of an operand tile's K step, into registers (zero outside the matrix or when
// `on` is false).  Both orientations run through the same two loads: only the addresses differ.
// Everything but the last few operations is uniform and stays on the scalar unit.  Returns whether
// the step is cut by the matrix edge inside a group of four (then the park has to zero the tails).
template <int TX>
__device__ __forceinline__ bool rb_fetch(Fetch& r, const RbLane& L, bool along_x, const float* P, long long sx, long long sk,
                                int x0, int Xe, int k0, int Ke, bool on) {
  const float* base = P + x0 * (along_x ? 1LL : sx) + k0 * (along_x ? sk : 1LL);
  const int cleft = along_x ? Xe - x0 : Ke - k0;          // extent left along the contiguous index
  const int sleft = on ? (along_x ? Ke - k0 : Xe - x0) : 0;  // and along the strided one
#pragma unroll
  for (int u = 0; u < 2; ++u) load_quad(r, u, base + L.off[u], (L.act[u] && L.s[u] < sleft) ? cleft - L.c[u] : 0);
  return (cleft & 3) != 0 && cleft < (along_x ? TX : RK);
}

// Zeroes the elements past the matrix edge of a fetched pair of groups.
__device__ __forceinline__ void trim_fetch(Fetch& r) {
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int j = 0; j < 4; ++j) r.q[u][j] = j < r.n[u] ? r.q[u][j] : 0.f;
}

template <int TX>
__device__ __forceinline__ void rb_park(RbTile<TX>& T, const Fetch& r, bool along_x, int tid) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef RbSplit<TX> S;
  if (along_x) {
    const int c = tid % S::combos, sh = tid / S::combos;
    if (sh < S::split) {
      const int xq = c % (TX / 4), ghf = c / (TX / 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float* dst = &T.v[ghf / 2][ghf % 2][rb_row(4 * xq + j)][S::NS * sh];
        if (S::NS == 2) *reinterpret_cast<f32x2*>(dst) = f32x2{r.q[0][j], r.q[1][j]};
        else *dst = r.q[0][j];
      }
    }
  } else {
    if (tid < S::items) {
      const int gq = tid % (RK / 8), x = tid / (RK / 8);
      *reinterpret_cast<f32x4*>(&T.v[gq][0][rb_row(x)][0]) = f32x4{r.q[0][0], r.q[0][2], r.q[1][0], r.q[1][2]};
      *reinterpret_cast<f32x4*>(&T.v[gq][1][rb_row(x)][0]) = f32x4{r.q[0][1], r.q[0][3], r.q[1][1], r.q[1][3]};
    }
  }
}

template <int WM, int WN, int BM, int BN>
struct RbShape {
  static constexpr int TM = 32 * BM * WM, TN = 32 * BN * WN;
  static constexpr size_t lds = 2 * (sizeof(RbTile<TM>) + sizeof(RbTile<TN>));
  static constexpr int per_cu = BM * BN >= 3 ? 3 : 4;  // resident workgroups the registers allow
};

// One output tile per workgroup (the hardware queue keeps three or four of them on a CU, so one tile's
// epilogue overlaps its neighbours' products).  The K steps are double-buffered: while step s is
// multiplied out of one LDS buffer, the elements of step s + 1 are on their way into registers, and they
// are parked in the other buffer, so there is one barrier per step.  Inside the loop nothing but the
// step's first-element pointers and remaining extents changes, all of it on the scalar unit.
template <int WM, int WN, int BM, int BN>
__global__ __launch_bounds__(256, (RbShape<WM, WN, BM, BN>::per_cu)) void k_gemm_rb(Gemm g) {
  static_assert(WM * WN == 4, "four waves");
  constexpr int TM = RbShape<WM, WN, BM, BN>::TM, TN = RbShape<WM, WN, BM, BN>::TN;
  extern __shared__ __attribute__((aligned(16))) unsigned char rb_smem[];
  RbTile<TM>* As = reinterpret_cast<RbTile<TM>*>(rb_smem);
  RbTile<TN>* Bs = reinterpret_cast<RbTile<TN>*>(rb_smem + 2 * sizeof(RbTile<TM>));
  const bool ax = g.modeA == GL_VEC_X, bx = g.modeB == GL_VEC_X;  // else GL_VEC_K

  GemmTile cur;
  if (!gemm_tile(g, blockIdx.x, (g.M + TM - 1) / TM, (g.N + TN - 1) / TN, TM, TN, cur)) return;

  typedef float f32x16 __attribute__((ext_vector_type(16)));
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x;
  const int lane = tid % 64, wv = __builtin_amdgcn_readfirstlane(tid / 64), l32 = lane % 32, hf = lane / 32;
  const int rbase = 32 * BM * (wv / WN), cbase = 32 * BN * (wv % WN);  // the wave's corner inside the tile
  const int row32 = rb_row(l32);

  // which of the wave's blocks do any work: inside the matrix and, for a triangular result, not
  // wholly above the diagonal
  bool work[BM][BN];
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j)
      work[i][j] = cur.m0 + rbase + 32 * i < cur.Me && cur.n0 + cbase + 32 * j < cur.Ne &&
                   !(g.mask == 1 && cur.n0 + cbase + 32 * j > cur.m0 + rbase + 32 * i + 31);

  f32x16 acc[BM][BN];
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // one product A B over its K steps, added into acc
  auto product = [&](const float* Ap, const float* Bp, long long sAm, long long sAk, long long sBn, long long sBk, int Ke,
                     bool a_x, bool b_x) {
    const RbLane la = rb_lane<TM>(a_x, sAm, sAk, tid), lb = rb_lane<TN>(b_x, sBn, sBk, tid);
    Fetch ra, rb;
    bool edge_a = rb_fetch<TM>(ra, la, a_x, Ap, sAm, sAk, cur.m0, cur.Me, 0, Ke, true);
    bool edge_b = rb_fetch<TN>(rb, lb, b_x, Bp, sBn, sBk, cur.n0, cur.Ne, 0, Ke, true);
    int buf = 0;
    // at least one step, so that an empty contraction still stores beta * C
    for (int k0 = 0; k0 == 0 || k0 < Ke; k0 += RK) {
      if (edge_a) trim_fetch(ra);
      if (edge_b) trim_fetch(rb);
      rb_park<TM>(As[buf], ra, a_x, tid);
      rb_park<TN>(Bs[buf], rb, b_x, tid);
      const bool more = k0 + RK < Ke;
      edge_a = rb_fetch<TM>(ra, la, a_x, Ap, sAm, sAk, cur.m0, cur.Me, k0 + RK, Ke, more);
      edge_b = rb_fetch<TN>(rb, lb, b_x, Bp, sBn, sBk, cur.n0, cur.Ne, k0 + RK, Ke, more);
      __syncthreads();
      const int ng = min(RK / 8, (Ke - k0 + 7) / 8);  // groups of eight k that hold data
      for (int gq = 0; gq < ng; ++gq) {
        f32x4 a[BM], b[BN];
#pragma unroll
        for (int i = 0; i < BM; ++i)
          a[i] = *reinterpret_cast<const f32x4*>(__builtin_assume_aligned(&As[buf].v[gq][hf][rbase + 32 * i + row32][0], 16));
#pragma unroll
        for (int j = 0; j < BN; ++j)
          b[j] = *reinterpret_cast<const f32x4*>(__builtin_assume_aligned(&Bs[buf].v[gq][hf][cbase + 32 * j + row32][0], 16));
#pragma unroll
        for (int i = 0; i < BM; ++i)
#pragma unroll
          for (int j = 0; j < BN; ++j)
            if (work[i][j]) {
#pragma unroll
              for (int s = 0; s < 4; ++s)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][s], b[j][s], acc[i][j], 0, 0, 0);
            }
      }
      buf ^= 1;
    }
  };
  product(cur.A, cur.B, g.sAm, g.sAk, g.sBn, g.sBk, cur.Ke, ax, bx);
  if (cur.xA != nullptr) {
    __syncthreads();  // the slower waves may still be reading the last step's buffer
    product(cur.xA, cur.xB, g.xsAm, g.xsAk, g.xsBn, g.xsBk, cur.xKe, g.xmodeA == GL_VEC_X, g.xmodeB == GL_VEC_X);
  }
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j)
      gemm_store_block(g, cur.C, cur.E, cur.m0 + rbase + 32 * i, hf, cur.Me, cur.n0 + cbase + 32 * j, l32, cur.Ne, acc[i][j]);
}

// dst[row][0..cols) = (float)src[row][0..cols);  dst[row][cols] = 1 if ones.
template <typename T>
__global__ void k_load_rows(const T* __restrict__ src, float* __restrict__ dst, long long rows, int cols, int ld,
                            int ones) {
  // threadIdx.x walks the columns, threadIdx.y the rows of the block: no index division
  const long long row = blockIdx.x * (long long)blockDim.y + threadIdx.y;
  if (row >= rows) return;
  for (int c = threadIdx.x; c < ld; c += blockDim.x)
    dst[row * ld + c] = c < cols ? load_as_f32(src, row * cols + c) : (ones ? 1.f : 0.f);
}

// Shift groups: the key-side stabilisers are per feature and per group of G consecutive positions of a
// (b,h) (G = L: one group per (b,h), the bidirectional case; G = the chunk length in the causal passes).
// Index of the group that holds `row` of a [B*H, L] row space.
__device__ __forceinline__ long long shift_group(long long row, int L, int G) {
  const long long bh = row / L;
  return bh * ((L + G - 1) / G) + (row - bh * L) / G;
}

// One wave per row: n = 1/2 |x~|^2, logits = U - n (+ bias_j) in place, rowmax.
// bias (optional): m per-feature shifts for every shift group (the key-side stabilisers,
// which the query side adds back so that every product phi_Q,j * phi_K,j is unchanged).
// exp_rows != 0: the row is left as exp(logit - rowmax) instead (the query features), the logits of up
// to 512 features staying in registers in between, so the row is read and written once.
// (V = 4: the row is walked in 16-byte groups; needs m % 4 == 0 and 16-byte aligned rows.)
template <int V>
__device__ __forceinline__ void load_v(const float* p, float (&o)[V]) {
  if (V == 4) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 x = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
    for (int e = 0; e < V; ++e) o[e] = x[e];
  } else {
    o[0] = p[0];
  }
}
template <int V>
__device__ __forceinline__ void store_v(float* p, const float (&o)[V]) {
  if (V == 4) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    *reinterpret_cast<f32x4*>(p) = f32x4{o[0], o[V > 1 ? 1 : 0], o[V > 2 ? 2 : 0], o[V > 3 ? 3 : 0]};
  } else {
    p[0] = o[0];
  }
}

template <int V>
__global__ __launch_bounds__(256) void k_rowstat(float* __restrict__ U, const float* __restrict__ Xt,
                                                 float* __restrict__ rowmax, const float* __restrict__ bias,
                                                 long long rows, int m, int r, int L, int exp_rows, int G) {
  constexpr int kKeep = 8 / (V == 4 ? 4 : 1);  // groups kept in registers: up to 512 features
  long long row = blockIdx.x * 4LL + threadIdx.x / kWave;
  if (row >= rows) return;
  int lane = threadIdx.x % kWave;
  const float* bs = bias ? bias + shift_group(row, L, G) * m : nullptr;
  const float* xt = Xt + row * r;
  float s = 0.f;
  for (int t = lane; t < r; t += kWave) s = fmaf(xt[t], xt[t], s);
  s = 0.5f * wave_sum(s);
  float* u = U + row * m;
  const int ng = m / V;  // groups in the row
  float mx = -INFINITY;
  float keep[kKeep][V];
#pragma unroll
  for (int t = 0; t < kKeep; ++t) {
    const int j = lane + kWave * t;
#pragma unroll
    for (int e = 0; e < V; ++e) keep[t][e] = -INFINITY;
    if (j < ng) {
      float b4[V];
      load_v<V>(u + V * j, keep[t]);
#pragma unroll
      for (int e = 0; e < V; ++e) b4[e] = 0.f;
      if (bs) load_v<V>(bs + V * j, b4);
#pragma unroll
      for (int e = 0; e < V; ++e) keep[t][e] = keep[t][e] - s + b4[e];
      if (!exp_rows) store_v<V>(u + V * j, keep[t]);
    }
#pragma unroll
    for (int e = 0; e < V; ++e) mx = fmaxf(mx, keep[t][e]);
  }
  for (int j = lane + kWave * kKeep; j < ng; j += kWave) {
    float v[V], b4[V];
    load_v<V>(u + V * j, v);
#pragma unroll
    for (int e = 0; e < V; ++e) b4[e] = 0.f;
    if (bs) load_v<V>(bs + V * j, b4);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      v[e] = v[e] - s + b4[e];
      mx = fmaxf(mx, v[e]);
    }
    store_v<V>(u + V * j, v);
  }
  mx = wave_max(mx);
  if (lane == 0) rowmax[row] = mx;
  if (exp_rows) {
#pragma unroll
    for (int t = 0; t < kKeep; ++t) {
      const int j = lane + kWave * t;
      if (j < ng) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) o[e] = expf(keep[t][e] - mx);
        store_v<V>(u + V * j, o);
      }
    }
    for (int j = lane + kWave * kKeep; j < ng; j += kWave) {
      float v[V];
      load_v<V>(u + V * j, v);
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] = expf(v[e] - mx);
      store_v<V>(u + V * j, v);
    }
  }
}

// One block per (b,h): maximum of L row maxima.
__global__ __launch_bounds__(256) void k_headmax(const float* __restrict__ rowmax, float* __restrict__ headmax, int L) {
  __shared__ float sm[4];
  const float* p = rowmax + (long long)blockIdx.x * L;
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < L; i += 256) mx = fmaxf(mx, p[i]);
  mx = wave_max(mx);
  if (threadIdx.x % kWave == 0) sm[threadIdx.x / kWave] = mx;
  __syncthreads();
  if (threadIdx.x == 0) headmax[blockIdx.x] = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
}

// Per-feature maximum over the rows of each shift group: colmax[group][j] = max over the group's rows l of
// logit[bh][l][j].  One block per (group, 64-column group); threads = 64 columns x 16 row phases, eight
// loads in flight.
constexpr int kColmaxPhases = 16;
// rown (optional): a per-row term subtracted from every entry first (the norm term n_l).
__global__ __launch_bounds__(64 * kColmaxPhases) void k_colmax(const float* __restrict__ logit,
                                                               float* __restrict__ colmax, int L, int m,
                                                               const float* __restrict__ rown, int G) {
  __shared__ float sm[kColmaxPhases][64];
  const int groups = (m + 63) / 64;
  const int ng = (L + G - 1) / G;
  const long long sg = blockIdx.x / groups;  // shift group
  const long long bh = sg / ng;
  const int l0 = (int)(sg % ng) * G, l1 = min(L, l0 + G);
  const int j = (blockIdx.x % groups) * 64 + threadIdx.x % 64;
  const int ph = threadIdx.x / 64;
  float mx = -INFINITY;
  if (j < m) {
    const float* p = logit + bh * L * (long long)m + j;
    const float* rn = rown ? rown + bh * L : nullptr;
    int l = l0 + ph;
    for (; l + 7 * kColmaxPhases < l1; l += 8 * kColmaxPhases) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(long long)(l + u * kColmaxPhases) * m];
      if (rn) {
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] -= rn[l + u * kColmaxPhases];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) mx = fmaxf(mx, v[u]);
    }
    for (; l < l1; l += kColmaxPhases) mx = fmaxf(mx, p[(long long)l * m] - (rn ? rn[l] : 0.f));
  }
  sm[ph][threadIdx.x % 64] = mx;
  __syncthreads();
  if (ph == 0 && j < m) {
#pragma unroll
    for (int u = 1; u < kColmaxPhases; ++u) mx = fmaxf(mx, sm[u][threadIdx.x]);
    colmax[sg * m + j] = mx;
  }
}

// Causal passes: the shift of a group becomes the maximum over the groups up to it (in place), so that a
// key is never stored under a shift set by keys that come after its chunk, and the shifts only grow along
// the sequence.  One thread per (b,h, feature); eight groups' values are loaded before the first is rewritten.
__global__ __launch_bounds__(256) void k_runmax(float* __restrict__ colmax, long long BH, int ng, int m) {
  const long long i = blockIdx.x * 256LL + threadIdx.x;
  if (i >= BH * m) return;
  float* p = colmax + (i / m) * ng * m + i % m;
  float run = -INFINITY;
  for (int g0 = 0; g0 < ng; g0 += 8) {
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = g0 + u < ng ? p[(long long)(g0 + u) * m] : -INFINITY;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      run = fmaxf(run, t[u]);
      if (g0 + u < ng) p[(long long)(g0 + u) * m] = run;
    }
  }
}

// Phi = exp(logit - c) * mult.  mode 0: c = cvec[row];  1: c = cvec[row / L] (per head);
// 2: c = cvec[group(row) * m + j] (per shift group of G positions and feature).
// rown (optional): a per-row term added to c (the norm term n_l, when the logits do not hold it yet).
// One wave per row, V features per lane and step (V = 4 needs m % 4 == 0 and 16-byte aligned rows).
template <typename T, int V>
__global__ __launch_bounds__(256) void k_exp(const float* __restrict__ logit, T* __restrict__ out,
                                             const float* __restrict__ cvec, long long rows, int m, int L, int mode,
                                             float mult, const float* __restrict__ rown, int G) {
  long long row = blockIdx.x * 4LL + threadIdx.x / kWave;
  if (row >= rows) return;
  const int lane = threadIdx.x % kWave;
  const float rn = rown ? rown[row] : 0.f;
  const float crow = (mode == 0 ? cvec[row] : (mode == 1 ? cvec[row / L] : 0.f)) + rn;
  const float* cj = mode == 2 ? cvec + shift_group(row, L, G) * m : nullptr;
  const float* src = logit + row * m;
  for (int j = lane; j < m / V; j += kWave) {
    float v[V], c[V];
    load_v<V>(src + V * j, v);
#pragma unroll
    for (int e = 0; e < V; ++e) c[e] = 0.f;
    if (cj) load_v<V>(cj + V * j, c);
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = expf(v[e] - (c[e] + crow)) * mult;
    if (sizeof(T) == 4) {
      store_v<V>(reinterpret_cast<float*>(out) + row * m + V * j, v);
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) store_from_f32(out, row * m + V * j + e, v[e]);
    }
  }
}

// n[row] = 1/2 |x~_row|^2, one wave per row.
__global__ __launch_bounds__(256) void k_rownorm(const float* __restrict__ Xt, float* __restrict__ n, long long rows, int r) {
  long long row = blockIdx.x * 4LL + threadIdx.x / kWave;
  if (row >= rows) return;
  int lane = threadIdx.x % kWave;
  const float* xt = Xt + row * r;
  float s = 0.f;
  for (int t = lane; t < r; t += kWave) s = fmaf(xt[t], xt[t], s);
  s = 0.5f * wave_sum(s);
  if (lane == 0) n[row] = s;
}

// out[o*so_out + e] = sum_{p<P} in[o*so + p*sp + e], p ascending (fixed order).
__global__ void k_sum_slices(const float* __restrict__ in, float* __restrict__ out, long long n_outer, int P,
                             long long E, long long so, long long sp) {
  long long total = n_outer * E;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    long long o = i / E, e = i % E;
    const float* q = in + o * so + e;
    float s = 0.f;
    for (int p = 0; p < P; ++p) s += q[p * sp];
    out[i] = s;
  }
}

// out[row][c] = ND[row][c] / ND[row][dv]
template <typename T>
__global__ void k_finish(const float* __restrict__ ND, T* __restrict__ out, long long rows, int dv, int ld) {
  long long total = rows * dv;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    long long row = i / dv;
    int c = (int)(i % dv);
    const float* nd = ND + row * ld;
    store_from_f32(out, i, nd[c] / nd[dv]);
  }
}

// Exclusive scan over the chunk axis of st[bh][chunk][E] (forward, or reverse for the
// backward pass), in place.  E = m * ld: row j of a chunk's state belongs to feature j and is expressed
// under that chunk's shift cm[bh][chunk][j] (running maxima: non-decreasing along the sequence).  What has
// been summed so far is brought to the shift of the chunk it is handed to before it is stored: forward, the
// sum over earlier chunks times exp(cm[c - 1] - cm[c]); reverse, the sum over later chunks times
// exp(cm[c] - cm[c + 1]) (there the states hold query features, which carry the shifts with the opposite
// sign).  Both factors are at most one.  cm == nullptr: plain sums.
__global__ void k_scan(float* __restrict__ st, long long BH, int nchunk, long long E, int reverse,
                       const float* __restrict__ cm, int m, int ld) {
  long long total = BH * E;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    long long bh = i / E, e = i % E;
    float* p = st + bh * nchunk * E + e;
    const float* cj = cm ? cm + bh * nchunk * m + e / ld : nullptr;
    float run = 0.f;
    float cprev = 0.f;  // shift of the chunk handled last
    // eight chunks' entries are loaded before the first is overwritten: the loads do not depend on the
    // running sum, but the compiler may not move them across the stores by itself
    constexpr int kBatch = 8;
    for (int c0 = 0; c0 < nchunk; c0 += kBatch) {
      float t[kBatch], cs[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int c = reverse ? nchunk - 1 - (c0 + u) : c0 + u;
        t[u] = c0 + u < nchunk ? p[c * E] : 0.f;
        cs[u] = cj && c0 + u < nchunk ? cj[(long long)c * m] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int c = reverse ? nchunk - 1 - (c0 + u) : c0 + u;
        if (c0 + u < nchunk) {
          if (cj && c0 + u > 0) run *= expf(reverse ? cs[u] - cprev : cprev - cs[u]);
          cprev = cs[u];
          p[c * E] = run;
          run += t[u];
        }
      }
    }
  }
}

// Backward, per row (one wave): from ND = [N | D] and G = dOut,
//   dN = G / D,  dD = -(G . out) / D  with out = N / D;  written as dND = [dN | dD].
template <typename T>
__global__ __launch_bounds__(256) void k_dnd(const float* __restrict__ ND, const T* __restrict__ G,
                                             float* __restrict__ dND, long long rows, int dv, int ld) {
  long long row = blockIdx.x * 4LL + threadIdx.x / kWave;
  if (row >= rows) return;
  int lane = threadIdx.x % kWave;
  const float* nd = ND + row * ld;
  float* o = dND + row * ld;
  float invD = 1.f / nd[dv];
  float dot = 0.f;
  for (int c = lane; c < dv; c += kWave) {
    float gv = load_as_f32(G, row * dv + c);
    o[c] = gv * invD;
    dot = fmaf(gv, nd[c] * invD, dot);
  }
  dot = wave_sum(dot);
  if (lane == 0) o[dv] = -dot * invD;
}

// Backward, per key row (one wave).  The logit gradients come out of the GEMMs already multiplied by the
// features.  What is left is the path through the norm term n = 1/2 |x~|^2, which enters every logit of
// the row with coefficient -1:  dn = -sum_j dlogit_j.  For a key row that sum is
// sum_j phi_K,lj (R_lj . [v_l | 1]) = [v_l | 1] . dVx_l, with dVx = Phi_K R over all dv + 1 columns (the
// first dv of them are dV), so it needs no pass over the m features.  For a query row the sum is
// N_i . dN_i + D_i dD_i = 0 identically (the output does not change when a query's features are all
// scaled alike), so the query side has no such term.
//   dXt = alpha dn * Xt (in place; alpha = sqrt(scale), the factor x~ carries from x' = sqrt(scale) x is
//   applied here so that the products that use dXt need no scale of their own), and dV = the first dv
//   columns of dVx if asked for.
__global__ __launch_bounds__(256) void k_key_dn(const float* __restrict__ Vx, const float* __restrict__ dVx,
                                                float* __restrict__ Xt, float* __restrict__ dV, long long rows, int dv,
                                                int ld, int r, float alpha) {
  long long row = blockIdx.x * 4LL + threadIdx.x / kWave;
  if (row >= rows) return;
  int lane = threadIdx.x % kWave;
  const float* vx = Vx + row * ld;
  const float* dx = dVx + row * ld;
  float s = 0.f;
  for (int c = lane; c <= dv; c += kWave) {
    const float g = dx[c];
    s = fmaf(vx[c], g, s);
    if (dV != nullptr && c < dv) dV[row * dv + c] = g;
  }
  const float dn = -alpha * wave_sum(s);
  float* xt = Xt + row * r;
  for (int t = lane; t < r; t += kWave) xt[t] *= dn;
}

// ------------------------------ host helpers -------------------------------
inline int grid_for(long long total, int block = 256) {
  long long g = (total + block - 1) / block;
  if (g > 65535LL * 16) g = 65535LL * 16;
  if (g < 1) g = 1;
  return (int)g;
}

Gemm gemm_base(const float* A, const float* B, float* C, int M, int N, int K) {
  Gemm g{};
  g.A = A;
  g.B = B;
  g.C = C;
  g.M = M;
  g.N = N;
  g.K = K;
  g.nb0 = g.nb1 = g.nb2 = 1;
  g.alpha = 1.f;
  g.beta = 0.f;
  return g;
}

// g += second product taken from the operand side of `x` (same M, N, batches and C as g).
void add_product(Gemm& g, const Gemm& x) {
  g.xA = x.A; g.xB = x.B; g.xK = x.K;
  g.xsAm = x.sAm; g.xsAk = x.sAk; g.xsBk = x.sBk; g.xsBn = x.sBn;
  g.xsA0 = x.sA0; g.xsA1 = x.sA1; g.xsA2 = x.sA2;
  g.xsB0 = x.sB0; g.xsB1 = x.sB1; g.xsB2 = x.sB2;
  g.xklim = x.klim; g.xkstep = x.kstep;
}

template <int WM, int WN, int BM, int BN>
dark_status launch_gemm_rb(const Gemm& g, hipStream_t st) {
  typedef RbShape<WM, WN, BM, BN> S;
  static bool granted = false;
  if (!granted) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_rb<WM, WN, BM, BN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::lds) != hipSuccess)
      return DARK_EHIP;
    granted = true;
  }
  const long long blocks = (long long)((g.M + S::TM - 1) / S::TM) * ((g.N + S::TN - 1) / S::TN) * g.nb0 * g.nb1 * g.nb2;
  if (blocks > 0x7fffffffLL) return DARK_EUNSUPPORTED;
  DARK_LAUNCH(KID_GEMM, st, (k_gemm_rb<WM, WN, BM, BN>), dim3((unsigned)blocks), dim3(256), S::lds, g);
  return DARK_OK;
}

dark_status run_gemm(const Gemm& g_in, hipStream_t st) {
  if ((long long)g_in.M * g_in.N * g_in.nb0 * g_in.nb1 * g_in.nb2 <= 0) return DARK_OK;
  Gemm g = g_in;
  g.modeA = gemm_load_mode(g.A, g.sAm, g.sAk, g.M, g.K, g.sA0, g.sA1, g.sA2);
  g.modeB = gemm_load_mode(g.B, g.sBn, g.sBk, g.N, g.K, g.sB0, g.sB1, g.sB2);
  if (g.xA != nullptr) {
    g.xmodeA = gemm_load_mode(g.xA, g.xsAm, g.xsAk, g.M, g.xK, g.xsA0, g.xsA1, g.xsA2);
    g.xmodeB = gemm_load_mode(g.xB, g.xsBn, g.xsBk, g.N, g.xK, g.xsB0, g.xsB1, g.xsB2);
    if (g.modeA == GL_SCALAR || g.modeB == GL_SCALAR || g.xmodeA == GL_SCALAR || g.xmodeB == GL_SCALAR) {
      // only the register-blocked kernel adds a second product: run it as a GEMM of its own
      Gemm first = g, second = g;
      first.xA = nullptr;
      first.E = nullptr;  // the element-wise factor multiplies the whole sum
      second.xA = nullptr;
      second.A = g.xA; second.B = g.xB; second.K = g.xK;
      second.sAm = g.xsAm; second.sAk = g.xsAk; second.sBk = g.xsBk; second.sBn = g.xsBn;
      second.sA0 = g.xsA0; second.sA1 = g.xsA1; second.sA2 = g.xsA2;
      second.sB0 = g.xsB0; second.sB1 = g.xsB1; second.sB2 = g.xsB2;
      second.klim = g.xklim; second.kstep = g.xkstep;
      second.beta = 1.f;  // alpha (A B + xA xB) + beta C  =  alpha xA xB + (alpha A B + beta C)
      DARK_TRY(run_gemm(first, st));
      return run_gemm(second, st);
    }
  }
  const bool vec = g.modeA != GL_SCALAR && g.modeB != GL_SCALAR;
  if (vec) {
    // The largest tile that still gives about as many tiles as the chip holds workgroups.
    const long long nb = (long long)g.nb0 * g.nb1 * g.nb2;
    auto enough = [&](int tm, int tn, int per_cu) {
      const long long tiles = (long long)((g.M + tm - 1) / tm) * ((g.N + tn - 1) / tn) * nb;
      return 4 * tiles >= 3 * 256LL * per_cu;
    };
    if (g.M > 64 && g.N > 96 && enough(128, 128, 3)) return launch_gemm_rb<2, 2, 2, 2>(g, st);
    if (g.M > 64 && g.N > 64 && g.N <= 96 && enough(128, 96, 3)) return launch_gemm_rb<4, 1, 1, 3>(g, st);
    if (g.M > 64 && enough(128, 64, 4)) return launch_gemm_rb<2, 2, 2, 1>(g, st);
    return launch_gemm_rb<2, 2, 1, 1>(g, st);
  }
  long long tiles = (long long)((g.M + GT - 1) / GT) * ((g.N + GT - 1) / GT);
  long long blocks = tiles * g.nb0 * g.nb1 * g.nb2;
  if (blocks <= 0) return DARK_OK;
  if (blocks > 0x7fffffffLL) return DARK_EUNSUPPORTED;
  // persistent workgroups, three per CU
  const unsigned grid = (unsigned)(blocks < 768 ? blocks : 768);
  DARK_LAUNCH(KID_GEMM, st, k_gemm, dim3(grid), dim3(256), 0, g, (int)blocks);
  return DARK_OK;
}

// Convert (or alias) an io tensor to fp32 rows with leading dimension ld.
dark_status to_f32(const Problem& pb, const void* src, float* dst, long long rows, int cols, int ld, int ones) {
  int tpr = 8;  // threads per row: the largest power of two not above ld, between 8 and 256
  while (tpr * 2 <= ld && tpr < 256) tpr *= 2;
  const dim3 block(tpr, 256 / tpr);
  const long long blocks = (rows + block.y - 1) / block.y;
  if (blocks > 0x7fffffffLL) return DARK_EUNSUPPORTED;
  if (blocks <= 0) return DARK_OK;
  if (pb.p.io_dtype == DARK_BF16)
    DARK_LAUNCH(KID_LOAD, pb.st, k_load_rows<__hip_bfloat16>, dim3((unsigned)blocks), block, 0,
                (const __hip_bfloat16*)src, dst, rows, cols, ld, ones);
  else
    DARK_LAUNCH(KID_LOAD, pb.st, k_load_rows<float>, dim3((unsigned)blocks), block, 0, (const float*)src, dst, rows, cols,
                ld, ones);
  return DARK_OK;
}

struct FeatBufs {
  float* Xf;      // [rows, d] fp32 copy of the input (or the input itself)
  float* Xt;      // [rows, r]  x~ = sqrt(scale) M x
  float* Phi;     // [rows, m]  logits, then features
  float* rowmax;  // [rows]
  float* headmax; // [BH]      per-head maximum (dark_featurize, keys)
  float* colmax;  // [BH, m]   per-feature maxima of the key logits (attention paths)
};

enum StabMode { STAB_QUERY_ROW = 0, STAB_KEY_HEAD = 1, STAB_KEY_FEATURE = 2 };

// A_s[h] = sqrt(scale) * W[h] M[h]   (Appendix B: omega~_j = M^T w_j), [H, m, d].
dark_status make_As(const Problem& pb, const float* M, const float* W, float* As) {
  const dark_params& p = pb.p;
  Gemm g = gemm_base(W, M, As, p.m, p.d, p.r);
  g.sAm = p.r; g.sAk = 1; g.sBk = p.d; g.sBn = 1; g.sCm = p.d; g.sCn = 1;
  g.nb1 = p.H;
  g.sA1 = p.w_shared ? 0 : (long long)p.m * p.r;
  g.sB1 = (long long)p.r * p.d;
  g.sC1 = (long long)p.m * p.d;
  g.alpha = std::sqrt(pb.scale);
  return run_gemm(g, pb.st);
}

// Logits and features of all rows of one input tensor (Section 4.1).
//   Xt  = sqrt(scale) X M^T;  U = X A_s^T;  logit = U - 1/2|Xt|^2;  Phi = exp(logit - c).
// Queries: c = row maximum (after adding `qbias`, if given).  Keys: c = maximum over the
// (b,h) slice (STAB_KEY_HEAD, the dark_featurize contract) or per feature over the slice
// (STAB_KEY_FEATURE, used inside attention where the query side adds the shifts back).
// G: positions per shift group of the per-feature key shifts (0 = L: one group per (b,h)); `running`: the
// shift of a group is the maximum over the groups up to it (the causal passes).
dark_status features(const Problem& pb, const FeatBufs& fb, const float* M, const float* As, StabMode mode,
                     const float* qbias = nullptr, bool exp_rows = false, int G = 0, bool running = false) {
  const dark_params& p = pb.p;
  const long long rows = pb.rows();
  const float alpha = std::sqrt(pb.scale);
  if (G <= 0) G = p.L;
  const int ng = (p.L + G - 1) / G;
  {
    Gemm g = gemm_base(fb.Xf, M, fb.Xt, p.L, p.r, p.d);
    g.sAm = p.d; g.sAk = 1; g.sBk = 1; g.sBn = p.d; g.sCm = p.r; g.sCn = 1;
    g.nb0 = p.B; g.nb1 = p.H;
    g.sA0 = (long long)p.H * p.L * p.d; g.sA1 = (long long)p.L * p.d;
    g.sB0 = 0; g.sB1 = (long long)p.r * p.d;
    g.sC0 = (long long)p.H * p.L * p.r; g.sC1 = (long long)p.L * p.r;
    g.alpha = alpha;
    DARK_TRY(run_gemm(g, pb.st));
  }
  {
    Gemm g = gemm_base(fb.Xf, As, fb.Phi, p.L, p.m, p.d);
    g.sAm = p.d; g.sAk = 1; g.sBk = 1; g.sBn = p.d; g.sCm = p.m; g.sCn = 1;
    g.nb0 = p.B; g.nb1 = p.H;
    g.sA0 = (long long)p.H * p.L * p.d; g.sA1 = (long long)p.L * p.d;
    g.sB0 = 0; g.sB1 = (long long)p.m * p.d;
    g.sC0 = (long long)p.H * p.L * p.m; g.sC1 = (long long)p.L * p.m;
    DARK_TRY(run_gemm(g, pb.st));
  }
  if (mode == STAB_KEY_FEATURE) {
    // The logits stay U: the norm term (kept in fb.rowmax, which this mode does not otherwise use) is
    // applied where they are read, by the per-feature maximum here and by exp_inplace.
    DARK_LAUNCH(KID_ROWSTAT, pb.st, k_rownorm, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, fb.Xt, fb.rowmax, rows, p.r);
    DARK_LAUNCH(KID_HEADMAX, pb.st, k_colmax, dim3((unsigned)(pb.BH() * ng * ((p.m + 63) / 64))), dim3(64 * kColmaxPhases),
                0, fb.Phi, fb.colmax, p.L, p.m, fb.rowmax, G);
    if (running && ng > 1)
      DARK_LAUNCH(KID_HEADMAX, pb.st, k_runmax, dim3((unsigned)((pb.BH() * p.m + 255) / 256)), dim3(256), 0, fb.colmax,
                  pb.BH(), ng, p.m);
    return DARK_OK;
  }
  const float* bias = mode == STAB_QUERY_ROW ? qbias : nullptr;
  if (p.m % 4 == 0 && ((reinterpret_cast<uintptr_t>(fb.Phi) | reinterpret_cast<uintptr_t>(bias)) & 15) == 0)
    DARK_LAUNCH(KID_ROWSTAT, pb.st, k_rowstat<4>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, fb.Phi, fb.Xt,
                fb.rowmax, bias, rows, p.m, p.r, p.L, exp_rows ? 1 : 0, G);
  else
    DARK_LAUNCH(KID_ROWSTAT, pb.st, k_rowstat<1>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, fb.Phi, fb.Xt,
                fb.rowmax, bias, rows, p.m, p.r, p.L, exp_rows ? 1 : 0, G);
  if (mode == STAB_KEY_HEAD)
    DARK_LAUNCH(KID_HEADMAX, pb.st, k_headmax, dim3((unsigned)pb.BH()), dim3(256), 0, fb.rowmax, fb.headmax, p.L);
  return DARK_OK;
}

dark_status exp_inplace(const Problem& pb, const FeatBufs& fb, StabMode mode, int G = 0) {
  const long long rows = pb.rows();
  if (G <= 0) G = pb.p.L;
  const float* c = mode == STAB_QUERY_ROW ? fb.rowmax : (mode == STAB_KEY_HEAD ? fb.headmax : fb.colmax);
  const float* rown = mode == STAB_KEY_FEATURE ? fb.rowmax : nullptr;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  if (pb.p.m % 4 == 0 && ((reinterpret_cast<uintptr_t>(fb.Phi) | reinterpret_cast<uintptr_t>(c)) & 15) == 0)
    DARK_LAUNCH(KID_EXP, pb.st, (k_exp<float, 4>), dim3(grid), dim3(256), 0, fb.Phi, fb.Phi, c, rows, pb.p.m, pb.p.L,
                (int)mode, 1.0f, rown, G);
  else
    DARK_LAUNCH(KID_EXP, pb.st, (k_exp<float, 1>), dim3(grid), dim3(256), 0, fb.Phi, fb.Phi, c, rows, pb.p.m, pb.p.L,
                (int)mode, 1.0f, rown, G);
  return DARK_OK;
}

// Length of the L-slices whose partial states are summed in a fixed order: short enough that a
// states GEMM (two 128-row tiles per (b,h, slice) at m = 256) has about a thousand workgroups, whole
// 64-token multiples, at least 256 and at most 4096.  A function of the shape only, so results stay
// reproducible.
int slice_len(const Problem& pb) {
  long long want = 1024 / (pb.BH() * 2 > 0 ? pb.BH() * 2 : 1);
  if (want < 1) want = 1;
  long long sl = (pb.p.L + want - 1) / want;
  sl = ((sl + 63) / 64) * 64;
  if (sl < 256) sl = 256;
  if (sl > 4096) sl = 4096;
  return (int)sl;
}

// Gradient with respect to the draws W (the parameters of a learned feature kernel): the logits depend on W
// through w_j^T x~ only, so dW[h][j][:] = sum over tokens of dlogit_j x~^T = alpha (dlogit^T X)[j][:] M_h^T
// = alpha T[j][:] M_h^T, summed over the batch in ascending order (and over heads when W is shared).
__global__ __launch_bounds__(256) void k_dw(const float* __restrict__ T, const float* __restrict__ M,
                                            float* __restrict__ dW, int nb, int H, int m, int r, int d, int w_shared,
                                            float alpha) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long per = (long long)m * r;
  if (i >= (w_shared ? 1 : H) * per) return;
  const int t = (int)(i % r), j = (int)((i / r) % m);
  const int h0 = w_shared ? 0 : (int)(i / per), h1 = w_shared ? H : h0 + 1;
  float acc = 0.f;
  for (int h = h0; h < h1; ++h)
    for (int b = 0; b < nb; ++b) {
      const float* Tr = T + (((size_t)b * H + h) * m + j) * d;
      const float* Mr = M + ((size_t)h * r + t) * d;
      float s0 = 0.f;
      for (int c = 0; c < d; ++c) s0 = fmaf(Tr[c], Mr[c], s0);
      acc += s0;
    }
  dW[i] = alpha * acc;
}

__global__ __launch_bounds__(256) void k_fill_identity(float* __restrict__ Mid, long long n, int d) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) Mid[i] = ((i / d) % d == i % d) ? 1.f : 0.f;
}

}  // namespace

dark_status launch_dw(const Problem& pb, const float* T, int nb, const float* M, float* dW) {
  const dark_params& p = pb.p;
  const long long n = (long long)(p.w_shared ? 1 : p.H) * p.m * p.r;
  DARK_LAUNCH(KID_BWD_ELEM, pb.st, k_dw, dim3(grid_for(n)), dim3(256), 0, T, M, dW, nb, p.H, p.m, p.r, p.d, p.w_shared,
              std::sqrt(pb.scale));
  return DARK_OK;
}

dark_status fill_identity(const Problem& pb, float* Mid) {
  const long long n = (long long)pb.p.H * pb.p.d * pb.p.d;
  DARK_LAUNCH(KID_LOAD, pb.st, k_fill_identity, dim3(grid_for(n)), dim3(256), 0, Mid, n, pb.p.d);
  return DARK_OK;
}

// ===========================================================================
// dark_featurize
// ===========================================================================
dark_status f32_featurize(const Problem& pb, Arena& ar, const void* X, const float* M, const float* W,
                          int is_query, void* phi, float* stab) {
  const dark_params& p = pb.p;
  const long long rows = pb.rows();
  FeatBufs fb{};
  float* As = ar.take<float>((size_t)p.H * p.m * p.d);
  fb.Xf = p.io_dtype == DARK_BF16 ? ar.take<float>((size_t)rows * p.d) : nullptr;
  fb.Xt = ar.take<float>((size_t)rows * p.r);
  fb.Phi = ar.take<float>((size_t)rows * p.m);
  fb.rowmax = ar.take<float>((size_t)rows);
  fb.headmax = ar.take<float>((size_t)pb.BH());
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;

  if (p.io_dtype == DARK_BF16)
    DARK_TRY(to_f32(pb, X, fb.Xf, rows, p.d, p.d, 0));
  else
    fb.Xf = const_cast<float*>(static_cast<const float*>(X));
  DARK_TRY(make_As(pb, M, W, As));
  DARK_TRY(features(pb, fb, M, As, is_query ? STAB_QUERY_ROW : STAB_KEY_HEAD));
  const float mult = 1.0f / std::sqrt((float)p.m);
  const float* cvec = is_query ? fb.rowmax : fb.headmax;
  {
    // phi is the caller's buffer: 16-byte aligned by contract, rows of m elements
    const unsigned grid = (unsigned)((rows + 3) / 4);
    const bool vec = p.m % 4 == 0 && (reinterpret_cast<uintptr_t>(fb.Phi) & 15) == 0;
    const int kmode = is_query ? 0 : 1;
    if (p.io_dtype == DARK_BF16) {
      if (vec)
        DARK_LAUNCH(KID_EXP, pb.st, (k_exp<__hip_bfloat16, 4>), dim3(grid), dim3(256), 0, fb.Phi, (__hip_bfloat16*)phi, cvec,
                    rows, p.m, p.L, kmode, mult, (const float*)nullptr, p.L);
      else
        DARK_LAUNCH(KID_EXP, pb.st, (k_exp<__hip_bfloat16, 1>), dim3(grid), dim3(256), 0, fb.Phi, (__hip_bfloat16*)phi, cvec,
                    rows, p.m, p.L, kmode, mult, (const float*)nullptr, p.L);
    } else {
      if (vec && (reinterpret_cast<uintptr_t>(phi) & 15) == 0)
        DARK_LAUNCH(KID_EXP, pb.st, (k_exp<float, 4>), dim3(grid), dim3(256), 0, fb.Phi, (float*)phi, cvec, rows, p.m, p.L,
                    kmode, mult, (const float*)nullptr, p.L);
      else
        DARK_LAUNCH(KID_EXP, pb.st, (k_exp<float, 1>), dim3(grid), dim3(256), 0, fb.Phi, (float*)phi, cvec, rows, p.m, p.L,
                    kmode, mult, (const float*)nullptr, p.L);
    }
  }
  if (stab != nullptr) {
    long long n = is_query ? rows : pb.BH();
    // plain copy through the sum kernel (P = 1)
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for(n)), dim3(256), 0, cvec, stab, 1LL, 1, n, n, n);
  }
  return DARK_OK;
}

// ===========================================================================
// forward attention (bidirectional and causal) and backward, fp32
// ===========================================================================
namespace {

// [V|1], [N|D], their gradients and the states have dv + 1 columns; their rows are padded to a multiple of
// four floats so that the GEMM can fetch them with 16-byte loads (the padding is never read as data).
inline int padded_ld(int cols) { return (cols + 3) & ~3; }

struct AttnBufs {
  float* As;
  FeatBufs q, k;
  float* Vx;      // [rows, dv+1] = [V | 1]
  float* part;    // bidirectional: [BH, P, m, dv+1] per-slice states
  float* SZ;      // bidirectional: [BH, m, dv+1];  causal: [BH, nchunk, m, dv+1] exclusive prefix states
  float* ND;      // [rows, dv+1] numerators and denominator
  float* Pm;      // causal: [BH, nchunk, C, C] masked score tiles
  int P, nchunk;
};

void plan_attn(const Problem& pb, Arena& ar, bool causal, bool keep_xt, AttnBufs& b) {
  const dark_params& p = pb.p;
  const long long rows = pb.rows();
  const int ldv = padded_ld(p.dv + 1);
  const bool conv = p.io_dtype == DARK_BF16;
  b.As = ar.take<float>((size_t)p.H * p.m * p.d);
  b.q.Xf = conv ? ar.take<float>((size_t)rows * p.d) : nullptr;
  b.k.Xf = conv ? ar.take<float>((size_t)rows * p.d) : nullptr;
  b.q.Xt = ar.take<float>((size_t)rows * p.r);
  b.k.Xt = keep_xt ? ar.take<float>((size_t)rows * p.r) : b.q.Xt;
  b.q.Phi = ar.take<float>((size_t)rows * p.m);
  b.k.Phi = ar.take<float>((size_t)rows * p.m);
  b.q.rowmax = ar.take<float>((size_t)rows);
  b.k.rowmax = ar.take<float>((size_t)rows);
  b.q.headmax = b.k.headmax = nullptr;
  b.nchunk = (p.L + pb.chunk - 1) / pb.chunk;
  b.q.colmax = b.k.colmax = ar.take<float>((size_t)pb.BH() * (causal ? b.nchunk : 1) * p.m);
  b.Vx = ar.take<float>((size_t)rows * ldv);
  b.ND = ar.take<float>((size_t)rows * ldv);
  b.P = (p.L + slice_len(pb) - 1) / slice_len(pb);
  if (causal) {
    b.part = nullptr;
    b.SZ = ar.take<float>((size_t)pb.BH() * b.nchunk * p.m * ldv);
    b.Pm = ar.take<float>((size_t)pb.BH() * b.nchunk * pb.chunk * pb.chunk);
  } else {
    b.part = ar.take<float>((size_t)pb.BH() * b.P * p.m * ldv);
    b.SZ = ar.take<float>((size_t)pb.BH() * p.m * ldv);
    b.Pm = nullptr;
  }
}

// Batch strides of a [B,H,L,cols] tensor split along L into pieces of `piece` rows.
inline void bhl(long long& s0, long long& s1, long long& s2, const dark_params& p, long long cols, int piece) {
  s0 = (long long)p.H * p.L * cols;
  s1 = (long long)p.L * cols;
  s2 = (long long)piece * cols;
}

// States: per piece (slice or chunk) of the sequence, Phi_piece^T X_piece  ->  dst[bh][piece][mm][ldd] (nn columns used).
Gemm make_piece_states(const Problem& pb, const float* Phi, int mm, const float* X, int nn, int ldx, float* dst, int ldd,
                       int piece, int npiece, float beta) {
  const dark_params& p = pb.p;
  Gemm g = gemm_base(Phi, X, dst, mm, nn, piece);
  g.sAm = 1; g.sAk = mm; g.sBk = ldx; g.sBn = 1; g.sCm = ldd; g.sCn = 1;
  g.nb0 = p.B; g.nb1 = p.H; g.nb2 = npiece;
  bhl(g.sA0, g.sA1, g.sA2, p, mm, piece);
  bhl(g.sB0, g.sB1, g.sB2, p, ldx, piece);
  g.sC2 = (long long)mm * ldd;
  g.sC1 = g.sC2 * npiece;
  g.sC0 = g.sC1 * p.H;
  g.klim = p.L; g.kstep = piece;
  g.beta = beta;
  return g;
}

dark_status piece_states(const Problem& pb, const float* Phi, int mm, const float* X, int nn, int ldx, float* dst,
                         int ldd, int piece, int npiece, float beta) {
  return run_gemm(make_piece_states(pb, Phi, mm, X, nn, ldx, dst, ldd, piece, npiece, beta), pb.st);
}

// Rows times a per-(b,h[,chunk]) matrix:  dst[rows_piece][nn] (+)= X_piece[rows][kk] * St(^T).
// st_t == false: St is [kk][nn] (row-major, leading dimension ld_st);  true: St is [nn][kk].
// batch_shared: St is indexed by the head only ([H, ...], e.g. A_s) instead of by (b, h).
Gemm make_rows_times_state(const Problem& pb, const float* X, int kk, int ldx, const float* St, int ld_st, bool st_t,
                           bool per_chunk, long long st_elems, float* dst, int nn, int ldd, int piece, int npiece,
                           float alpha, float beta, bool batch_shared = false) {
  const dark_params& p = pb.p;
  Gemm g = gemm_base(X, St, dst, piece, nn, kk);
  g.sAm = ldx; g.sAk = 1;
  if (st_t) { g.sBk = 1; g.sBn = ld_st; } else { g.sBk = ld_st; g.sBn = 1; }
  g.sCm = ldd; g.sCn = 1;
  g.nb0 = p.B; g.nb1 = p.H; g.nb2 = npiece;
  bhl(g.sA0, g.sA1, g.sA2, p, ldx, piece);
  bhl(g.sC0, g.sC1, g.sC2, p, ldd, piece);
  g.sB2 = per_chunk ? st_elems : 0;
  g.sB1 = per_chunk ? st_elems * npiece : st_elems;
  g.sB0 = batch_shared ? 0 : g.sB1 * p.H;
  g.mlim = p.L; g.mstep = piece;
  g.alpha = alpha; g.beta = beta;
  return g;
}

dark_status rows_times_state(const Problem& pb, const float* X, int kk, int ldx, const float* St, int ld_st, bool st_t,
                             bool per_chunk, long long st_elems, float* dst, int nn, int ldd, int piece, int npiece,
                             float alpha, float beta, bool batch_shared = false) {
  return run_gemm(make_rows_times_state(pb, X, kk, ldx, St, ld_st, st_t, per_chunk, st_elems, dst, nn, ldd, piece, npiece,
                                        alpha, beta, batch_shared),
                  pb.st);
}

// Score-like tiles per chunk:  T[bh][c][i][l] = sum_k X[cC+i][k] Y[cC+l][k], lower-triangular.
dark_status chunk_tiles(const Problem& pb, const float* X, int ldx, const float* Y, int ldy, int kk, float* T) {
  const dark_params& p = pb.p;
  const int C = pb.chunk;
  const int nchunk = (p.L + C - 1) / C;
  Gemm g = gemm_base(X, Y, T, C, C, kk);
  g.sAm = ldx; g.sAk = 1; g.sBk = 1; g.sBn = ldy; g.sCm = C; g.sCn = 1;
  g.nb0 = p.B; g.nb1 = p.H; g.nb2 = nchunk;
  bhl(g.sA0, g.sA1, g.sA2, p, ldx, C);
  bhl(g.sB0, g.sB1, g.sB2, p, ldy, C);
  g.sC2 = (long long)C * C; g.sC1 = g.sC2 * nchunk; g.sC0 = g.sC1 * p.H;
  g.mlim = p.L; g.mstep = C; g.nlim = p.L; g.nstep = C;
  g.mask = 1;
  return run_gemm(g, pb.st);
}

// dst_chunk[rows][nn] += T_chunk(^T) [rows][C] * X_chunk[C][nn].
Gemm make_tile_times_rows(const Problem& pb, const float* T, bool transpose, const float* X, int ldx, float* dst,
                          int nn, int ldd) {
  const dark_params& p = pb.p;
  const int C = pb.chunk;
  const int nchunk = (p.L + C - 1) / C;
  Gemm g = gemm_base(T, X, dst, C, nn, C);
  if (transpose) { g.sAm = 1; g.sAk = C; } else { g.sAm = C; g.sAk = 1; }
  g.sBk = ldx; g.sBn = 1; g.sCm = ldd; g.sCn = 1;
  g.nb0 = p.B; g.nb1 = p.H; g.nb2 = nchunk;
  g.sA2 = (long long)C * C; g.sA1 = g.sA2 * nchunk; g.sA0 = g.sA1 * p.H;
  bhl(g.sB0, g.sB1, g.sB2, p, ldx, C);
  bhl(g.sC0, g.sC1, g.sC2, p, ldd, C);
  g.mlim = p.L; g.mstep = C; g.klim = p.L; g.kstep = C;
  g.beta = 1.f;
  return g;
}

// dst_chunk = rows-times-state product + tile-times-rows product, one pass over dst: `first` as built
// by make_rows_times_state (per chunk, beta = 0), `second` by make_tile_times_rows for the same dst.
dark_status run_chunk_pair(const Problem& pb, Gemm first, const Gemm& second) {
  add_product(first, second);
  return run_gemm(first, pb.st);
}

// Everything the forward pass computes up to ND = [numerator | denominator].
dark_status forward_core(const Problem& pb, AttnBufs& b, bool causal, const void* Q, const void* K, const void* V,
                         const float* M, const float* W) {
  const dark_params& p = pb.p;
  const long long rows = pb.rows();
  const int dv1 = p.dv + 1, ldv = padded_ld(dv1);
  if (p.io_dtype == DARK_BF16) {
    DARK_TRY(to_f32(pb, Q, b.q.Xf, rows, p.d, p.d, 0));
    DARK_TRY(to_f32(pb, K, b.k.Xf, rows, p.d, p.d, 0));
  } else {
    b.q.Xf = const_cast<float*>(static_cast<const float*>(Q));
    b.k.Xf = const_cast<float*>(static_cast<const float*>(K));
  }
  DARK_TRY(to_f32(pb, V, b.Vx, rows, p.dv, ldv, 1));
  DARK_TRY(make_As(pb, M, W, b.As));
  // Keys first: phi_K,lj = exp(logit_lj - c_j), c_j the per-feature maximum over the head.  The
  // queries add c_j back (phi_Q,ij = exp(logit_ij + c_j - rowmax_i)), so every product
  // phi_Q,ij phi_K,lj is the unshifted one times a per-row factor that cancels in N / D.
  // Causal: c_j is kept per chunk, the maximum over the chunks up to it, so that no key is stored under a
  // shift set by later keys (a query sees nothing of them); the states of earlier chunks are brought to
  // the chunk's shifts where they are added up (k_scan), by factors exp(c_earlier - c_later) <= 1.
  const int G = causal ? pb.chunk : 0;
  DARK_TRY(features(pb, b.k, M, b.As, STAB_KEY_FEATURE, nullptr, false, G, causal));
  DARK_TRY(exp_inplace(pb, b.k, STAB_KEY_FEATURE, G));
  DARK_TRY(features(pb, b.q, M, b.As, STAB_QUERY_ROW, b.k.colmax, true, G));  // leaves the query features
  const long long st_elems = (long long)p.m * ldv;
  if (!causal) {
    // [S|z] = Phi_K^T [V|1]: per-slice partial states, then a fixed-order sum (Section 2: K'^T V first).
    DARK_TRY(piece_states(pb, b.k.Phi, p.m, b.Vx, dv1, ldv, b.part, ldv, slice_len(pb), b.P, 0.f));
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for(pb.BH() * st_elems)), dim3(256), 0, b.part, b.SZ,
                pb.BH(), b.P, st_elems, st_elems * b.P, st_elems);
    // [N|D] = Phi_Q [S|z]   (then left-multiplying by Q')
    DARK_TRY(rows_times_state(pb, b.q.Phi, p.m, p.m, b.SZ, ldv, false, false, st_elems, b.ND, dv1, ldv, p.L, 1, 1.f,
                              0.f));
  } else {
    const int C = pb.chunk;
    DARK_TRY(piece_states(pb, b.k.Phi, p.m, b.Vx, dv1, ldv, b.SZ, ldv, C, b.nchunk, 0.f));
    DARK_LAUNCH(KID_SCAN, pb.st, k_scan, dim3(grid_for(pb.BH() * st_elems)), dim3(256), 0, b.SZ, pb.BH(), b.nchunk,
                st_elems, 0, (const float*)b.k.colmax, p.m, ldv);
    // inter-chunk: Phi_Q,c [S|z]_{<c};  intra-chunk: tril(Phi_Q,c Phi_K,c^T) [V_c|1]
    DARK_TRY(chunk_tiles(pb, b.q.Phi, p.m, b.k.Phi, p.m, p.m, b.Pm));
    DARK_TRY(run_chunk_pair(pb,
                            make_rows_times_state(pb, b.q.Phi, p.m, p.m, b.SZ, ldv, false, true, st_elems, b.ND, dv1, ldv,
                                                  C, b.nchunk, 1.f, 0.f),
                            make_tile_times_rows(pb, b.Pm, false, b.Vx, ldv, b.ND, dv1, ldv)));
  }
  return DARK_OK;
}

}  // namespace

dark_status f32_attn_fwd(const Problem& pb, Arena& ar, bool causal, const void* Q, const void* K, const void* V,
                         const float* M, const float* W, void* out) {
  AttnBufs b{};
  plan_attn(pb, ar, causal, false, b);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;
  DARK_TRY(forward_core(pb, b, causal, Q, K, V, M, W));
  const long long rows = pb.rows();
  if (pb.p.out_dtype == DARK_BF16)
    DARK_LAUNCH(KID_FINISH, pb.st, k_finish<__hip_bfloat16>, dim3(grid_for(rows * pb.p.dv)), dim3(256), 0, b.ND,
                (__hip_bfloat16*)out, rows, pb.p.dv, padded_ld(pb.p.dv + 1));
  else
    DARK_LAUNCH(KID_FINISH, pb.st, k_finish<float>, dim3(grid_for(rows * pb.p.dv)), dim3(256), 0, b.ND, (float*)out,
                rows, pb.p.dv, padded_ld(pb.p.dv + 1));
  return DARK_OK;
}

// Backward.  With G = dOut, N_i / D_i the numerator / denominator of out_i and the
// (prefix) states S_i, z_i:
//   dN_i = G_i / D_i,   dD_i = -(G_i . out_i) / D_i
//   R_l  = sum_{i >= l} Phi_Q,i [dN_i | dD_i]^T            (all i if bidirectional)
//   dV_l = R_l[:, :dv]^T Phi_K,l
//   dPhi_Q,i = [S_i | z_i] [dN_i | dD_i]^T,   dPhi_K,l = R_l [v_l | 1]^T
//   dlogit = dPhi * Phi (applied in the epilogue of the GEMM that forms dPhi)
//   dn_l = -sum_j dlogit_K,lj = -[v_l | 1] . (R_l^T Phi_K,l),  dXt_K = sqrt(scale) dn Xt_K;  the query rows have dn = 0
//   dQ = dlogit_Q A_s,   dK = dlogit_K A_s + dXt_K M
//   dM_h = sum_b ( sqrt(scale) W^T (dlogit_Q^T Q + dlogit_K^T K) + dXt_K^T K )
// Stabilising shifts cancel between dPhi and Phi, so the stabilised features are used
// throughout.  Causal: states are exclusive prefix (S) / suffix (R) sums over chunks plus
// masked within-chunk tiles  P = tril(Phi_Q Phi_K^T),  E = tril([dN|dD] [V|1]^T).
dark_status f32_attn_bwd(const Problem& pb, Arena& ar, bool causal, const void* Q, const void* K, const void* V,
                         const float* M, const float* W, const void* dOut, float* dQ, float* dK, float* dV,
                         float* dM, float* dW) {
  const dark_params& p = pb.p;
  const long long rows = pb.rows();
  const int dv1 = p.dv + 1, ldv = padded_ld(dv1);
  const int C = pb.chunk;
  AttnBufs b{};
  plan_attn(pb, ar, causal, true, b);
  const long long st_elems = (long long)p.m * ldv;
  float* dND = ar.take<float>((size_t)rows * ldv);
  float* dPq = ar.take<float>((size_t)rows * p.m);
  float* dPk = ar.take<float>((size_t)rows * p.m);
  float* dVx = ar.take<float>((size_t)rows * ldv);  // Phi_K R over all dv + 1 columns
  float* R = ar.take<float>((size_t)pb.BH() * (causal ? b.nchunk : 1) * st_elems);
  float* Rpart = causal ? nullptr : ar.take<float>((size_t)pb.BH() * b.P * st_elems);
  float* Em = causal ? ar.take<float>((size_t)pb.BH() * b.nchunk * C * C) : nullptr;
  float* Tpart = ar.take<float>((size_t)pb.BH() * b.P * p.m * p.d);
  float* T = ar.take<float>((size_t)pb.BH() * p.m * p.d);
  float* T2part = ar.take<float>((size_t)pb.BH() * b.P * p.r * p.d);
  float* T2 = ar.take<float>((size_t)pb.BH() * p.r * p.d);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;

  DARK_TRY(forward_core(pb, b, causal, Q, K, V, M, W));
  if (p.io_dtype == DARK_BF16)
    DARK_LAUNCH(KID_BWD_ELEM, pb.st, k_dnd<__hip_bfloat16>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, b.ND,
                (const __hip_bfloat16*)dOut, dND, rows, p.dv, ldv);
  else
    DARK_LAUNCH(KID_BWD_ELEM, pb.st, k_dnd<float>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, b.ND,
                (const float*)dOut, dND, rows, p.dv, ldv);
  // dVx feeds dV and, through the key norms, dK and dM
  const bool need_dvx = dV != nullptr || dK != nullptr || dM != nullptr;

  if (!causal) {
    DARK_TRY(piece_states(pb, b.q.Phi, p.m, dND, dv1, ldv, Rpart, ldv, slice_len(pb), b.P, 0.f));
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for(pb.BH() * st_elems)), dim3(256), 0, Rpart, R,
                pb.BH(), b.P, st_elems, st_elems * b.P, st_elems);
    Gemm gq = make_rows_times_state(pb, dND, dv1, ldv, b.SZ, ldv, true, false, st_elems, dPq, p.m, p.m, p.L, 1, 1.f, 0.f);
    gq.E = b.q.Phi;
    DARK_TRY(run_gemm(gq, pb.st));
    Gemm gk = make_rows_times_state(pb, b.Vx, dv1, ldv, R, ldv, true, false, st_elems, dPk, p.m, p.m, p.L, 1, 1.f, 0.f);
    gk.E = b.k.Phi;
    DARK_TRY(run_gemm(gk, pb.st));
    if (need_dvx)
      DARK_TRY(rows_times_state(pb, b.k.Phi, p.m, p.m, R, ldv, false, false, st_elems, dVx, dv1, ldv, p.L, 1, 1.f, 0.f));
  } else {
    DARK_TRY(piece_states(pb, b.q.Phi, p.m, dND, dv1, ldv, R, ldv, C, b.nchunk, 0.f));
    DARK_LAUNCH(KID_SCAN, pb.st, k_scan, dim3(grid_for(pb.BH() * st_elems)), dim3(256), 0, R, pb.BH(), b.nchunk,
                st_elems, 1, (const float*)b.k.colmax, p.m, ldv);
    DARK_TRY(chunk_tiles(pb, dND, ldv, b.Vx, ldv, dv1, Em));  // E_il = dN_i . v_l + dD_i, l <= i
    // b.Pm = tril(Phi_Q Phi_K^T) is left over from forward_core.
    Gemm gq = make_rows_times_state(pb, dND, dv1, ldv, b.SZ, ldv, true, true, st_elems, dPq, p.m, p.m, C, b.nchunk, 1.f,
                                    0.f);
    gq.E = b.q.Phi;
    DARK_TRY(run_chunk_pair(pb, gq, make_tile_times_rows(pb, Em, false, b.k.Phi, p.m, dPq, p.m, p.m)));
    Gemm gk = make_rows_times_state(pb, b.Vx, dv1, ldv, R, ldv, true, true, st_elems, dPk, p.m, p.m, C, b.nchunk, 1.f,
                                    0.f);
    gk.E = b.k.Phi;
    DARK_TRY(run_chunk_pair(pb, gk, make_tile_times_rows(pb, Em, true, b.q.Phi, p.m, dPk, p.m, p.m)));
    if (need_dvx)
      DARK_TRY(run_chunk_pair(pb,
                              make_rows_times_state(pb, b.k.Phi, p.m, p.m, R, ldv, false, true, st_elems, dVx, dv1, ldv,
                                                    C, b.nchunk, 1.f, 0.f),
                              make_tile_times_rows(pb, b.Pm, true, dND, ldv, dVx, dv1, ldv)));
  }
  // dPq / dPk hold the logit gradients; dXt_K (in the key Xt buffer) and dV
  if (need_dvx)
    DARK_LAUNCH(KID_BWD_ELEM, pb.st, k_key_dn, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, b.Vx, dVx, b.k.Xt, dV, rows,
                p.dv, ldv, p.r, std::sqrt(pb.scale));
  const float alpha = std::sqrt(pb.scale);
  const long long as_elems = (long long)p.m * p.d, m_elems = (long long)p.r * p.d;
  for (int side = 0; side < 2; ++side) {
    float* dX = side == 0 ? dQ : dK;
    if (!dX) continue;
    float* dl = side == 0 ? dPq : dPk;
    Gemm g = make_rows_times_state(pb, dl, p.m, p.m, b.As, p.d, false, false, as_elems, dX, p.d, p.d, p.L, 1, 1.f, 0.f,
                                   true);
    if (side == 1) {
      // the norm term (keys only): + dXt_K M, with M [H, r, d] shared over the batch
      Gemm x = gemm_base(b.k.Xt, M, dX, p.L, p.d, p.r);
      x.sAm = p.r; x.sAk = 1; x.sBk = p.d; x.sBn = 1;
      x.sA0 = (long long)p.H * p.L * p.r; x.sA1 = (long long)p.L * p.r;
      x.sB0 = 0; x.sB1 = m_elems;
      add_product(g, x);
    }
    DARK_TRY(run_gemm(g, pb.st));
  }
  if (dM || dW) {
    const int SL = slice_len(pb);
    {  // Tpart = dlogit_Q^T Q + dlogit_K^T K per slice, one pass
      Gemm g = make_piece_states(pb, dPq, p.m, b.q.Xf, p.d, p.d, Tpart, p.d, SL, b.P, 0.f);
      add_product(g, make_piece_states(pb, dPk, p.m, b.k.Xf, p.d, p.d, Tpart, p.d, SL, b.P, 0.f));
      DARK_TRY(run_gemm(g, pb.st));
    }
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for(pb.BH() * as_elems)), dim3(256), 0, Tpart, T,
                pb.BH(), b.P, as_elems, as_elems * b.P, as_elems);
    if (dW) DARK_TRY(launch_dw(pb, T, p.B, M, dW));
  }
  if (dM) {
    const int SL = slice_len(pb);
    DARK_TRY(piece_states(pb, b.k.Xt, p.r, b.k.Xf, p.d, p.d, T2part, p.d, SL, b.P, 0.f));
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for(pb.BH() * m_elems)), dim3(256), 0, T2part, T2,
                pb.BH(), b.P, m_elems, m_elems * b.P, m_elems);
    // T2_bh = alpha * W_h^T T_bh + T2_bh
    Gemm g = gemm_base(W, T, T2, p.r, p.d, p.m);
    g.sAm = 1; g.sAk = p.r; g.sBk = p.d; g.sBn = 1; g.sCm = p.d; g.sCn = 1;
    g.nb0 = p.B; g.nb1 = p.H;
    g.sA0 = 0; g.sA1 = p.w_shared ? 0 : (long long)p.m * p.r;
    g.sB0 = as_elems * p.H; g.sB1 = as_elems;
    g.sC0 = m_elems * p.H; g.sC1 = m_elems;
    g.alpha = alpha; g.beta = 1.f;  // dXt carries its factor already
    DARK_TRY(run_gemm(g, pb.st));
    // dM_h = sum_b T2_bh, b ascending
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_sum_slices, dim3(grid_for((long long)p.H * m_elems)), dim3(256), 0, T2, dM,
                (long long)p.H, p.B, m_elems, m_elems, m_elems * p.H);
  }
  return DARK_OK;
}

}  // namespace dark

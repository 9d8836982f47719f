// Whitening geometry: M = Lambda^{-1/2} from the rows of Q and K (Section 4.1 of the paper: with input
// covariance Lambda, Sigma = Lambda^{-1} whitens the inputs; Proposition C.1: M = Lambda^{-1/2} makes
// Cov(M q) = I).  An initialiser for the learned geometry, computed once per model, not per step.
//
//   k_moments_mfma / k_moments   per (head, chunk of rows): sum of x x^T and of x        (HBM-bound: one read of Q, K)
//   k_moments_sum                per head: fixed-order fp64 sum of the chunks, centred covariance Lambda
//   k_whiten_eig                 per head: eigen-decomposition of Lambda by parallel cyclic Jacobi rotations in
//                                LDS, M = diag(lambda^-1/2) U^T for the r directions of largest variance
// Readings (the paper gives no estimator): Q and K are pooled (it assumes Cov(q) = Cov(k), Section 3); the
// covariance is the centred sample covariance with divisor N; eigenvalues below kFloor times the largest are
// raised to it; rows of M are ordered by decreasing variance (any rotation of the rows gives the same Sigma).
#include <cmath>

#include "fused_common.h"

namespace dark {
using namespace fz;
namespace {

constexpr float kFloor = 1e-6f;
constexpr int kChunkRows = 1024;  // rows of one (tensor, b) per workgroup

// ---------------------------------------------------------------------------
// k_moments_mfma (bf16, d = 64 or 128): tiles of 64 rows go to LDS as they are; the d x d sum of outer
// products is X^T X by 32x32x16 bf16 MFMAs whose two operands are both transposing reads of the tile
// (products of bf16 values are exact in fp32).  Wave w owns the 32 x 32 blocks b with b % 4 == w.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32x4 frag_tr(const unsigned short* base, int ld, int k0, int n0, int lane) {
  // fragment of a tile stored [k][n], n contiguous: lane (l32, hf) gets elements k0 + 8 hf + [0,8) of column
  // n0 + l32, by two 4 x 16 transposing reads
  const int l16 = lane % 16, grp = lane / 16;
  const unsigned short* p = base + (k0 + 8 * (grp / 2) + l16 / 4) * ld + n0 + 16 * (grp % 2) + 4 * (l16 % 4);
  const u32x2 lo = lds_read_tr16(p);
  const u32x2 hi = lds_read_tr16(p + 4 * ld);
  return u32x4{lo[0], lo[1], hi[0], hi[1]};
}

template <int D>
__global__ __launch_bounds__(256) void k_moments_mfma(const unsigned short* __restrict__ Qg,
                                                      const unsigned short* __restrict__ Kg, float* __restrict__ part,
                                                      int B, int H, int L, int chunks_per_seq, int ntensor) {
  constexpr int LD = D + 8, TT = 64, NB = D / 32, NBLK = NB * NB / 4;  // blocks per wave: 1 or 4
  __shared__ __attribute__((aligned(16))) unsigned short Xs[2][TT * LD];
  const int tid = threadIdx.x, lane = tid % 64, wv = tid / 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int nchunk = ntensor * B * chunks_per_seq;
  const int h = blockIdx.x / nchunk, ck = blockIdx.x % nchunk;
  const int tensor = ck / (B * chunks_per_seq), b = (ck / chunks_per_seq) % B, cs = ck % chunks_per_seq;
  const unsigned short* X = (tensor == 0 ? Qg : Kg) + ((size_t)b * H + h) * L * D;
  const int row0 = cs * kChunkRows, row1 = min(L, row0 + kChunkRows);
  const int ntile = (row1 - row0 + TT - 1) / TT;
  constexpr int PIECES = TT * D / 8 / 256;  // 16-byte pieces per thread and tile: 2 or 4
  // three tiles of rows are in flight in registers (the kernel has nothing to do but wait for memory)
  constexpr int AHEAD = 3;
  u32x4 reg[AHEAD][PIECES];
  auto fetch = [&](int t, u32x4(&rg)[PIECES]) {
#pragma unroll
    for (int u = 0; u < PIECES; ++u) {
      const int ci = tid + 256 * u, r = ci / (D / 8), kc = ci % (D / 8);
      const int row = row0 + t * TT + r;
      rg[u] = row < row1 ? *reinterpret_cast<const u32x4*>(X + (size_t)row * D + 8 * kc) : u32x4{0u, 0u, 0u, 0u};
    }
  };
  auto commit = [&](int buf, const u32x4(&rg)[PIECES]) {
#pragma unroll
    for (int u = 0; u < PIECES; ++u) {
      const int ci = tid + 256 * u, r = ci / (D / 8), kc = ci % (D / 8);
      *reinterpret_cast<u32x4*>(&Xs[buf][r * LD + 8 * kc]) = rg[u];
    }
  };
  f32x16 acc[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  float csum = 0.f;
#pragma unroll
  for (int a = 0; a < AHEAD; ++a)
    if (a < ntile) fetch(a, reg[a]);
  // the register sets rotate with the tile index: the loop is unrolled by AHEAD so that the indices are static
  for (int t0 = 0; t0 < ntile; t0 += AHEAD) {
#pragma unroll
  for (int a = 0; a < AHEAD; ++a) {
    const int t = t0 + a;
    if (t >= ntile) break;
    commit(t % 2, reg[a]);
    if (t + AHEAD < ntile) fetch(t + AHEAD, reg[a]);
    __syncthreads();  // also separates this tile's reads from the commit two tiles later
    const unsigned short* xs = Xs[t % 2];
#pragma unroll
    for (int s = 0; s < TT / 16; ++s) {
#pragma unroll
      for (int i = 0; i < NBLK; ++i) {
        const int blk = wv + 4 * i, rb = blk / NB, cb = blk % NB;
        const u32x4 a = frag_tr(xs, LD, 16 * s, 32 * rb, lane), bq = frag_tr(xs, LD, 16 * s, 32 * cb, lane);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(const_cast<u32x4*>(&a)),
                                                         *reinterpret_cast<bf16x8*>(const_cast<u32x4*>(&bq)), acc[i], 0, 0, 0);
      }
    }
    if (tid < D) {
      float a = 0.f;
#pragma unroll 8
      for (int r = 0; r < TT; ++r) a += __uint_as_float((unsigned)xs[r * LD + tid] << 16);
      csum += a;
    }
  }
  }
  float* out = part + (size_t)blockIdx.x * (D * D + D);
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    const int blk = wv + 4 * i, rb = blk / NB, cb = blk % NB;
#pragma unroll
    for (int v = 0; v < 16; ++v) out[(32 * rb + 8 * (v / 4) + 4 * hf + (v % 4)) * D + 32 * cb + l32] = acc[i][v];
  }
  if (tid < D) out[D * D + tid] = csum;
}

// ---------------------------------------------------------------------------
// k_moments (any dtype, d <= 128): the same sums on the vector ALU.  Thread (ti, tj) of a 16 x 16 grid owns the
// entries (ti + 16 a, tj + 16 b); tiles of 32 rows sit in LDS as fp32.
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float ld_f32(const T* p, size_t i);
template <>
__device__ __forceinline__ float ld_f32<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ld_f32<unsigned short>(const unsigned short* p, size_t i) {
  return __uint_as_float((unsigned)p[i] << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void k_moments(const T* __restrict__ Qg, const T* __restrict__ Kg,
                                                 float* __restrict__ part, int B, int H, int L, int d,
                                                 int chunks_per_seq, int ntensor) {
  constexpr int TT = 32, MAXA = 8;  // d <= 128
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* xs = reinterpret_cast<float*>(smem);  // [TT][d + 1]
  const int ld = d + 1;
  const int tid = threadIdx.x, ti = tid / 16, tj = tid % 16;
  const int nchunk = ntensor * B * chunks_per_seq;
  const int h = blockIdx.x / nchunk, ck = blockIdx.x % nchunk;
  const int tensor = ck / (B * chunks_per_seq), b = (ck / chunks_per_seq) % B, cs = ck % chunks_per_seq;
  const T* X = (tensor == 0 ? Qg : Kg) + ((size_t)b * H + h) * L * d;
  const int row0 = cs * kChunkRows, row1 = min(L, row0 + kChunkRows);
  const int na = (d + 15) / 16;
  float acc[MAXA][MAXA];
#pragma unroll
  for (int a = 0; a < MAXA; ++a)
#pragma unroll
    for (int c = 0; c < MAXA; ++c) acc[a][c] = 0.f;
  float csum = 0.f;
  for (int t0 = row0; t0 < row1; t0 += TT) {
    __syncthreads();
    for (int i = tid; i < TT * d; i += 256) {
      const int r = i / d, c = i % d;
      xs[r * ld + c] = t0 + r < row1 ? ld_f32<T>(X, (size_t)(t0 + r) * d + c) : 0.f;
    }
    __syncthreads();
    for (int r = 0; r < TT; ++r) {
      float xi[MAXA], xj[MAXA];
#pragma unroll
      for (int a = 0; a < MAXA; ++a) {
        xi[a] = (a < na && ti + 16 * a < d) ? xs[r * ld + ti + 16 * a] : 0.f;
        xj[a] = (a < na && tj + 16 * a < d) ? xs[r * ld + tj + 16 * a] : 0.f;
      }
#pragma unroll
      for (int a = 0; a < MAXA; ++a)
#pragma unroll
        for (int c = 0; c < MAXA; ++c) acc[a][c] = fmaf(xi[a], xj[c], acc[a][c]);
    }
    if (tid < d) {
      float a = 0.f;
      for (int r = 0; r < TT; ++r) a += xs[r * ld + tid];
      csum += a;
    }
  }
  float* out = part + (size_t)blockIdx.x * ((size_t)d * d + d);
#pragma unroll
  for (int a = 0; a < MAXA; ++a)
#pragma unroll
    for (int c = 0; c < MAXA; ++c) {
      const int i = ti + 16 * a, j = tj + 16 * c;
      if (i < d && j < d) out[(size_t)i * d + j] = acc[a][c];
    }
  if (tid < d) out[(size_t)d * d + tid] = csum;
}

// ---------------------------------------------------------------------------
// k_moments_sum: Lambda[h] = (Sxx - Sx Sx^T / N) / N, the chunk sums added in ascending order in fp64.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_moments_sum(const float* __restrict__ part, float* __restrict__ cov, int H,
                                                     int d, int nchunk, double nrows) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)H * d * d) return;
  const int h = (int)(idx / ((long long)d * d)), e = (int)(idx % ((long long)d * d));
  const int i = e / d, j = e % d;
  const size_t per = (size_t)d * d + d;
  const float* base = part + (size_t)h * nchunk * per;
  double sxx = 0.0, si = 0.0, sj = 0.0;
  for (int c0 = 0; c0 < nchunk; c0 += 8) {
    float a[8], bi[8], bj[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const size_t o = (size_t)min(c0 + u, nchunk - 1) * per;
      a[u] = base[o + e];
      bi[u] = base[o + (size_t)d * d + i];
      bj[u] = base[o + (size_t)d * d + j];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (c0 + u < nchunk) {
        sxx += (double)a[u];
        si += (double)bi[u];
        sj += (double)bj[u];
      }
  }
  cov[idx] = (float)((sxx - si * sj / nrows) / nrows);
}

// ---------------------------------------------------------------------------
// k_whiten_eig: one workgroup per head.  A = Lambda and V = I in LDS (fp32); sweeps of parallel cyclic Jacobi:
// in each of the n - 1 steps of a sweep the n / 2 disjoint index pairs of a round-robin schedule are rotated
// at once (angles from the current 2 x 2 blocks, then all row updates, then all column updates of A and V).
// Jacobi rotations keep the relative accuracy of small eigenvalues of a graded positive definite matrix, which
// is what the inverse square root needs.  Stops when no off-diagonal entry exceeds 2e-5 sqrt(a_pp a_qq) (rounding in fp32 leaves about 6e-8 sqrt(condition number) there, and Sigma is then
// accurate to about that figure; the eigenvalues are converged to second order in it), or
// after kMaxSweeps.
// ---------------------------------------------------------------------------
constexpr int kMaxSweeps = 16;
__global__ __launch_bounds__(1024) void k_whiten_eig(const float* __restrict__ cov, float* __restrict__ M, int d, int r) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int ld = d + 1;
  float* A = reinterpret_cast<float*>(smem);
  float* V = A + (size_t)d * ld;
  float* cs = V + (size_t)d * ld;            // [n/2][2]
  int* pq = reinterpret_cast<int*>(cs + d + 2);  // [n/2][2]
  float* lam = reinterpret_cast<float*>(pq + d + 2);  // [d]
  int* order = reinterpret_cast<int*>(lam + d);       // [d]
  __shared__ unsigned offmax;
  const int tid = threadIdx.x, h = blockIdx.x;
  const int n = d + (d & 1), np = n / 2;
  for (int i = tid; i < d * d; i += 1024) {
    A[(i / d) * ld + i % d] = cov[(size_t)h * d * d + i];
    V[(i / d) * ld + i % d] = (i / d == i % d) ? 1.f : 0.f;
  }
  __syncthreads();
  for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
    if (tid == 0) offmax = 0u;
    for (int s = 0; s < n - 1; ++s) {
      __syncthreads();
      if (tid < np) {
        int p, q;
        if (tid == 0) {
          p = n - 1;
          q = s;
        } else {
          p = (s + tid) % (n - 1);
          q = (s - tid + (n - 1)) % (n - 1);
        }
        if (p > q) {
          const int t = p;
          p = q;
          q = t;
        }
        float c = 1.f, sn = 0.f;
        if (q < d) {  // an odd d plays against a dummy index
          const float app = A[p * ld + p], aqq = A[q * ld + q], apq = A[p * ld + q];
          const float rel = fabsf(apq) / fmaxf(sqrtf(fabsf(app * aqq)), 1e-37f);
          atomicMax(&offmax, __float_as_uint(rel));
          if (apq != 0.f && rel > 1e-9f) {
            const float tau = (aqq - app) / (2.f * apq);
            const float tt = (tau >= 0.f ? 1.f : -1.f) / (fabsf(tau) + sqrtf(1.f + tau * tau));
            c = 1.f / sqrtf(1.f + tt * tt);
            sn = tt * c;
          }
        } else {
          q = -1;
        }
        cs[2 * tid] = c;
        cs[2 * tid + 1] = sn;
        pq[2 * tid] = p;
        pq[2 * tid + 1] = q;
      }
      __syncthreads();
      // rows p, q of A:  a_pj <- c a_pj - s a_qj,  a_qj <- s a_pj + c a_qj
      for (int i = tid; i < np * d; i += 1024) {
        const int k = i / d, j = i % d, p = pq[2 * k], q = pq[2 * k + 1];
        if (q >= 0) {
          const float c = cs[2 * k], sn = cs[2 * k + 1];
          const float x = A[p * ld + j], y = A[q * ld + j];
          A[p * ld + j] = c * x - sn * y;
          A[q * ld + j] = sn * x + c * y;
        }
      }
      __syncthreads();
      // columns p, q of A and of V
      for (int i = tid; i < np * d; i += 1024) {
        const int k = i / d, j = i % d, p = pq[2 * k], q = pq[2 * k + 1];
        if (q >= 0) {
          const float c = cs[2 * k], sn = cs[2 * k + 1];
          const float x = A[j * ld + p], y = A[j * ld + q];
          A[j * ld + p] = c * x - sn * y;
          A[j * ld + q] = sn * x + c * y;
          const float vx = V[j * ld + p], vy = V[j * ld + q];
          V[j * ld + p] = c * vx - sn * vy;
          V[j * ld + q] = sn * vx + c * vy;
        }
      }
    }
    __syncthreads();
    if (__uint_as_float(offmax) < 2e-5f) break;  // uniform: every thread reads the same word after the barrier
    __syncthreads();
  }
  __syncthreads();
  // eigenvalues in descending order (ties by index), floored
  if (tid < d) lam[tid] = A[tid * ld + tid];
  __syncthreads();
  if (tid < d) {
    const float mine = lam[tid];
    int rank = 0;
    for (int j = 0; j < d; ++j) rank += (lam[j] > mine || (lam[j] == mine && j < tid)) ? 1 : 0;
    order[rank] = tid;
  }
  __syncthreads();
  const float lmax = fmaxf(lam[order[0]], 1e-37f);
  for (int i = tid; i < r * d; i += 1024) {
    const int t = i / d, c = i % d, src = order[t];
    const float l = fmaxf(lam[src], kFloor * lmax);
    M[((size_t)h * r + t) * d + c] = V[c * ld + src] / sqrtf(l);
  }
}

size_t eig_lds(int d) {
  return (size_t)2 * d * (d + 1) * 4 + (size_t)(d + 2) * 4 * 2 + (size_t)d * 4 * 2 + 64;
}

}  // namespace

bool whiten_supported(const Problem& pb) {
  const dark_params& p = pb.p;
  return p.d <= 128 && p.r <= p.d;
}

dark_status whiten(const Problem& pb, Arena& ar, const void* Q, const void* K, float* M, float* cov_out) {
  const dark_params& p = pb.p;
  const int ntensor = K != nullptr || ar.base == nullptr ? 2 : 1;
  const int chunks_per_seq = (p.L + kChunkRows - 1) / kChunkRows;
  const int nchunk = 2 * p.B * chunks_per_seq;  // planned for two tensors, whether or not K is given
  const size_t per = (size_t)p.d * p.d + p.d;
  float* part = ar.take<float>((size_t)p.H * nchunk * per);
  float* cov = ar.take<float>((size_t)p.H * p.d * p.d);
  if (ar.base == nullptr) return DARK_OK;
  if (ar.overflow) return DARK_EWORKSPACE;
  if (cov_out != nullptr) cov = cov_out;
  const int used = ntensor * p.B * chunks_per_seq;
  const unsigned grid = (unsigned)(p.H * used);
  if (p.io_dtype == DARK_BF16 && (p.d == 64 || p.d == 128)) {
    if (p.d == 64)
      DARK_LAUNCH(KID_WHITEN_MOMENTS, pb.st, k_moments_mfma<64>, dim3(grid), dim3(256), 0, (const unsigned short*)Q,
                  (const unsigned short*)K, part, p.B, p.H, p.L, chunks_per_seq, ntensor);
    else
      DARK_LAUNCH(KID_WHITEN_MOMENTS, pb.st, k_moments_mfma<128>, dim3(grid), dim3(256), 0, (const unsigned short*)Q,
                  (const unsigned short*)K, part, p.B, p.H, p.L, chunks_per_seq, ntensor);
  } else {
    const size_t lds = (size_t)32 * (p.d + 1) * 4;
    if (p.io_dtype == DARK_BF16)
      DARK_LAUNCH(KID_WHITEN_MOMENTS, pb.st, k_moments<unsigned short>, dim3(grid), dim3(256), lds,
                  (const unsigned short*)Q, (const unsigned short*)K, part, p.B, p.H, p.L, p.d, chunks_per_seq, ntensor);
    else
      DARK_LAUNCH(KID_WHITEN_MOMENTS, pb.st, k_moments<float>, dim3(grid), dim3(256), lds, (const float*)Q,
                  (const float*)K, part, p.B, p.H, p.L, p.d, chunks_per_seq, ntensor);
  }
  {
    const long long n = (long long)p.H * p.d * p.d;
    DARK_LAUNCH(KID_SUM_SLICES, pb.st, k_moments_sum, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, part, cov, p.H,
                p.d, used, (double)ntensor * p.B * p.L);
  }
  const size_t lds = eig_lds(p.d);
  DARK_TRY(allow_lds(k_whiten_eig, lds));
  DARK_LAUNCH(KID_WHITEN_EIG, pb.st, k_whiten_eig, dim3((unsigned)p.H), dim3(1024), lds, cov, M, p.d, p.r);
  return DARK_OK;
}

}  // namespace dark

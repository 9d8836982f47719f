// One step of causal random-feature attention as a recurrence: the state (S, z) of a (b,h) absorbs the new
// key/value pair and the new query reads it out (the causal form of Section 2's linear attention, one token
// at a time: out_t = phi(q_t)^T S_t / phi(q_t)^T z_t with S_t = S_{t-1} + phi(k_t) v_t^T, z_t = z_{t-1} + phi(k_t)).
// The state is kept under one scalar shift c per (b,h) (natural-log domain): it holds sum_l exp(logit_l - c) v_l^T;
// a new key whose largest logit exceeds c raises c and rescales the state.
// One workgroup per (b,h); fp32 arithmetic; the step is bound by reading and writing the state once.
#include <cmath>

#include "common.h"

namespace dark {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ float ld1(const T* p, size_t i);
template <>
__device__ __forceinline__ float ld1<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ld1<unsigned short>(const unsigned short* p, size_t i) {
  return __uint_as_float((unsigned)p[i] << 16);
}
__device__ __forceinline__ void st1(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st1(unsigned short* p, size_t i, float v) {
  // round to nearest even
  unsigned u = __float_as_uint(v);
  if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
  p[i] = (unsigned short)(u >> 16);
}

__device__ __forceinline__ float block_max(float v, float* red, int tid) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  __syncthreads();
  if (tid % 64 == 0) red[tid / 64] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}
__device__ __forceinline__ float block_sum(float v, float* red, int tid) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if (tid % 64 == 0) red[tid / 64] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// LDS: xq[d], xk[d], tq[r], tk[r], eq[m], ek[m], vv[dv], num[256] (partial numerators), red[4]
template <typename T>
__global__ __launch_bounds__(256) void k_decode_step(const T* __restrict__ q, const T* __restrict__ k,
                                                     const T* __restrict__ v, const float* __restrict__ M,
                                                     const float* __restrict__ W, float* __restrict__ S,
                                                     float* __restrict__ z, float* __restrict__ c, T* __restrict__ out,
                                                     int H, int d, int r, int m, int dv, int w_shared, float alpha) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* xq = reinterpret_cast<float*>(smem);
  float* xk = xq + d;
  float* tq = xk + d;
  float* tk = tq + r;
  float* eq = tk + r;
  float* ek = eq + m;
  float* vv = reinterpret_cast<float*>(smem) + ((2 * d + 2 * r + 2 * m + 3) / 4) * 4;   // 16-byte aligned
  float* num = vv + ((dv + 3) / 4) * 4;      // [256]
  float* red = num + 256;    // [4]
  const int tid = threadIdx.x, bh = blockIdx.x, h = bh % H;
  // The state does not depend on anything computed here: when it is small enough (16 pieces of 16 bytes per
  // thread: m dv <= 16384) all of it is requested first and arrives while the logits are being formed.
  const int cg = (dv + 3) / 4;             // groups of four columns
  float* Sb = S + (size_t)bh * m * dv;
  float* zb = z + (size_t)bh * m;
  const bool vec = dv % 4 == 0 && 256 % cg == 0;
  const int col = vec ? 4 * (tid % cg) : 0, rstep = vec ? 256 / cg : 1;
  const bool early = vec && m <= 16 * rstep;
  f32x4 se[16];
  if (early) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int j = tid / cg + u * rstep;
      if (j < m) se[u] = *reinterpret_cast<const f32x4*>(Sb + (size_t)j * dv + col);
    }
  }
  for (int i = tid; i < d; i += 256) {
    xq[i] = alpha * ld1<T>(q, (size_t)bh * d + i);
    xk[i] = alpha * ld1<T>(k, (size_t)bh * d + i);
  }
  for (int i = tid; i < dv; i += 256) vv[i] = ld1<T>(v, (size_t)bh * dv + i);
  __syncthreads();
  // x~ = M x'
  const float* Mh = M != nullptr ? M + (size_t)h * r * d : nullptr;  // null: the identity (r == d)
  for (int t = tid; t < r; t += 256) {
    float a = 0.f, b = 0.f;
    if (Mh != nullptr && d % 4 == 0) {   // rows of M as 16-byte loads, eight in flight
      const f32x4* mr = reinterpret_cast<const f32x4*>(Mh + (size_t)t * d);
      for (int e0 = 0; e0 < d / 4; e0 += 8) {
        f32x4 mv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) mv[u] = mr[min(e0 + u, d / 4 - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (e0 + u < d / 4) {
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              a = fmaf(mv[u][x], xq[4 * (e0 + u) + x], a);
              b = fmaf(mv[u][x], xk[4 * (e0 + u) + x], b);
            }
          }
      }
    } else if (Mh != nullptr) {
      for (int e = 0; e < d; ++e) {
        const float mv = Mh[(size_t)t * d + e];
        a = fmaf(mv, xq[e], a);
        b = fmaf(mv, xk[e], b);
      }
    } else {
      a = xq[t];
      b = xk[t];
    }
    tq[t] = a;
    tk[t] = b;
  }
  __syncthreads();
  float nq = 0.f, nk = 0.f;
  for (int t = tid; t < r; t += 256) {
    nq = fmaf(tq[t], tq[t], nq);
    nk = fmaf(tk[t], tk[t], nk);
  }
  nq = 0.5f * block_sum(nq, red, tid);
  nk = 0.5f * block_sum(nk, red, tid);
  // logits
  const float* Wh = W + (w_shared ? 0 : (size_t)h * m * r);
  float mq = -INFINITY, mk = -INFINITY;
  for (int j = tid; j < m; j += 256) {
    float a = 0.f, b = 0.f;
    if (r % 4 == 0) {
      const f32x4* wr = reinterpret_cast<const f32x4*>(Wh + (size_t)j * r);
      for (int t0 = 0; t0 < r / 4; t0 += 8) {
        f32x4 wv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) wv[u] = wr[min(t0 + u, r / 4 - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (t0 + u < r / 4) {
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              a = fmaf(wv[u][x], tq[4 * (t0 + u) + x], a);
              b = fmaf(wv[u][x], tk[4 * (t0 + u) + x], b);
            }
          }
      }
    } else {
      for (int t = 0; t < r; ++t) {
        const float wv = Wh[(size_t)j * r + t];
        a = fmaf(wv, tq[t], a);
        b = fmaf(wv, tk[t], b);
      }
    }
    a -= nq;
    b -= nk;
    eq[j] = a;
    ek[j] = b;
    mq = fmaxf(mq, a);
    mk = fmaxf(mk, b);
  }
  mq = block_max(mq, red, tid);
  mk = block_max(mk, red, tid);
  const float c_old = c[bh];
  const float c_new = fmaxf(c_old, mk);
  const float down = expf(c_old - c_new);   // 0 for the first token (c_old = -inf)
  for (int j = tid; j < m; j += 256) {
    eq[j] = expf(eq[j] - mq);
    ek[j] = expf(ek[j] - c_new);
  }
  __syncthreads();
  // state update and read-out: thread t walks the rows j = t / cg, t / cg + 256 / cg, ... of its column group
  float den = 0.f;
  for (int j = tid; j < m; j += 256) {
    const float zn = zb[j] * down + ek[j];
    zb[j] = zn;
    den = fmaf(eq[j], zn, den);
  }
  den = block_sum(den, red, tid);
  const float inv = 1.f / den;
  if (vec) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const f32x4 v4 = *reinterpret_cast<const f32x4*>(vv + col);
    if (early) {
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int j = tid / cg + u * rstep;
        if (j < m) {
          const float e = ek[j], f = eq[j];
          f32x4 sn;
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            sn[x] = fmaf(e, v4[x], se[u][x] * down);
            acc[x] = fmaf(f, sn[x], acc[x]);
          }
          *reinterpret_cast<f32x4*>(Sb + (size_t)j * dv + col) = sn;
        }
      }
    } else
    for (int j0 = tid / cg; j0 < m; j0 += 4 * rstep) {
      f32x4 sv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (j0 + u * rstep < m) sv[u] = *reinterpret_cast<const f32x4*>(Sb + (size_t)(j0 + u * rstep) * dv + col);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int j = j0 + u * rstep;
        if (j < m) {
          const float e = ek[j], f = eq[j];
          f32x4 sn;
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            sn[x] = fmaf(e, v4[x], sv[u][x] * down);
            acc[x] = fmaf(f, sn[x], acc[x]);
          }
          *reinterpret_cast<f32x4*>(Sb + (size_t)j * dv + col) = sn;
        }
      }
    }
    // add the partial numerators of the threads that share a column group
    __syncthreads();
    for (int x = 0; x < 4; ++x) {
      num[tid] = acc[x];
      __syncthreads();
      if (tid < cg) {
        float s = 0.f;
        for (int u = tid; u < 256; u += cg) s += num[u];
        st1(out, (size_t)bh * dv + 4 * tid + x, s * inv);
      }
      __syncthreads();
    }
  } else {
    // general shapes: a thread per column
    for (int col = tid; col < dv; col += 256) {
      float acc = 0.f;
      for (int j = 0; j < m; ++j) {
        const float sn = fmaf(ek[j], vv[col], Sb[(size_t)j * dv + col] * down);
        Sb[(size_t)j * dv + col] = sn;
        acc = fmaf(eq[j], sn, acc);
      }
      st1(out, (size_t)bh * dv + col, acc * inv);
    }
  }
  if (tid == 0) c[bh] = c_new;
}

}  // namespace

dark_status decode_step(const Problem& pb, const void* q, const void* k, const void* v, const float* M,
                        const float* W, float* S, float* z, float* c, void* out) {
  const dark_params& p = pb.p;
  const size_t lds = (size_t)(2 * p.d + 2 * p.r + 2 * p.m + p.dv + 8 + 256 + 4) * sizeof(float);
  if (lds > 48 * 1024) return DARK_EUNSUPPORTED;
  const unsigned grid = (unsigned)pb.BH();
  const float alpha = std::sqrt(pb.scale);
  if (p.io_dtype == DARK_BF16)
    DARK_LAUNCH(KID_DECODE, pb.st, k_decode_step<unsigned short>, dim3(grid), dim3(256), lds, (const unsigned short*)q,
                (const unsigned short*)k, (const unsigned short*)v, M, W, S, z, c, (unsigned short*)out, p.H, p.d, p.r,
                p.m, p.dv, p.w_shared, alpha);
  else
    DARK_LAUNCH(KID_DECODE, pb.st, k_decode_step<float>, dim3(grid), dim3(256), lds, (const float*)q, (const float*)k,
                (const float*)v, M, W, S, z, c, (float*)out, p.H, p.d, p.r, p.m, p.dv, p.w_shared, alpha);
  return DARK_OK;
}

}  // namespace dark

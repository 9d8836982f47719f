// Device helpers and host-side hooks shared by the fused MFMA translation units (gfx950).
// Every translation unit that includes this header is compiled with -fno-honor-nans.
#pragma once

#include "common.h"

namespace dark {
namespace fz {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
// Running shifts are only raised when a feature value would exceed 2^kTau (rare): fp32 sums of such
// values over up to 2^20 positions, times the readout's own 2^kTau, stay far below 2^127.
constexpr float kTau = 40.0f;
constexpr float kBig = 1.099511627776e12f;  // 2^40
constexpr float kRaise = 20.0f;             // in the rare path, shifts more than 2^20 too low are raised
constexpr int kTile = 64;      // tokens per tile in the K pass
// The readout's fast path accepts a tile when every denominator lies in this range: numerators are
// bounded by max|v| times the denominator, so nothing has overflowed, and nothing was flushed.
constexpr float kDenLo = 7.888609052210118e-31f;  // 2^-100
constexpr float kDenHi = 7.922816251426434e28f;   // 2^96

__device__ static inline unsigned pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;
  p[1] = (__bf16)b;
  return *reinterpret_cast<unsigned*>(&p);
}
__device__ static inline unsigned pack_f16_from_bf16pair(unsigned w) {
  // w holds two bf16.  Magnitudes in [2^-14, 65504] convert exactly (8 significand bits fit in 11); smaller
  // ones lose bits to fp16's subnormals and vanish below 2^-25 (absolute error at most 2^-25 per element);
  // larger ones become +-inf (round to nearest), so that the result is visibly non-finite instead of
  // silently that of a clamped input.
  fp16x2 h;
  h[0] = (__fp16)__uint_as_float(w << 16);
  h[1] = (__fp16)__uint_as_float(w & 0xffff0000u);
  return *reinterpret_cast<unsigned*>(&h);
}
__device__ static inline u32x4 bf16x8_to_f16x8(u32x4 r) {
  u32x4 o;
  o[0] = pack_f16_from_bf16pair(r[0]);
  o[1] = pack_f16_from_bf16pair(r[1]);
  o[2] = pack_f16_from_bf16pair(r[2]);
  o[3] = pack_f16_from_bf16pair(r[3]);
  return o;
}
__device__ static inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// acc + a.lo * b.lo + a.hi * b.hi on packed bf16 pairs, fp32 arithmetic (v_dot2_f32_bf16)
__device__ static inline float dot2_bf16(unsigned a, unsigned b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(*reinterpret_cast<bf16x2*>(&a), *reinterpret_cast<bf16x2*>(&b), acc, false);
}
constexpr unsigned kOnesBf16x2 = 0x3f803f80u;
// max(a, b, c).  This file is compiled with -fno-honor-nans, so the compiler needs no NaN
// canonicalisation and forms v_max3_f32.  (Not inline asm: the compiler must see the reads of
// MFMA results to insert the wait states they need.)
__device__ static inline float max3(float a, float b, float c) { return __builtin_fmaxf(a, __builtin_fmaxf(b, c)); }
// Sum over each row of 16 lanes (result in every lane of the row): four DPP row rotations.
template <int N>
__device__ static inline float dpp_row_ror(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}
__device__ static inline float row16_sum(float v) {
  v += dpp_row_ror<8>(v);
  v += dpp_row_ror<4>(v);
  v += dpp_row_ror<2>(v);
  v += dpp_row_ror<1>(v);
  return v;
}


// ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the LDS address of four
// consecutive 16-bit values r_i[0..3]; lane l of the group receives r_{4e + l/4}[l % 4] for
// e = 0..3.  With lane i pointing at row i/4, columns 4 (i%4) .. 4 (i%4) + 3 of a row-major tile,
// lane l receives column l of rows 0..3: a 4 x 16 transpose.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ static inline u32x2 lds_read_tr16(const unsigned short* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(const_cast<unsigned short*>(p)));
  return *reinterpret_cast<u32x2*>(&v);
}

// The value of lane l ^ 32 / l ^ 16, by the lane-swap instructions of gfx950 (vector ALU, no trip through the LDS
// crossbar as __shfl_xor takes).  v_permlane32_swap exchanges the upper half of its first operand with the lower
// half of the second; v_permlane16_swap does the same with the odd rows of 16 lanes of the first and the even rows
// of the second.  With both operands the same value, the second result of the former and the first... see below.
__device__ static inline float xor32(float v) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {lower: own lower, upper: own lower}; r[1] = {lower: own upper, upper: own upper}
  return __uint_as_float(threadIdx.x & 32 ? r[0] : r[1]);
}
__device__ static inline float xor16(float v) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  // rows of 16 lanes: r[0] = {even rows: own, odd rows: the even row below}; r[1] = {even rows: the odd row above, odd rows: own}
  return __uint_as_float(threadIdx.x & 16 ? r[0] : r[1]);
}

// XOR swizzle of the 16-byte chunks of a row of a bf16 V tile in LDS (ROWB bytes per row: 64 or 128 value columns):
// chunk q of row `row` sits at position q ^ v_swz<ROWB>(row).  The transposing reads of the products phi^T V fetch,
// per group of 16 lanes, two neighbouring chunks of four consecutive rows; rows of 128 (256) bytes fall onto the
// same banks every second row (every row), and with this choice the 32 lanes that the LDS serves together find their
// 32 eight-byte words on 32 different bank pairs (2.4 cycles per instruction, the rate of a contiguous read;
// XOR with the row number itself: 4 cycles at 128-byte rows, 8 at 256-byte rows).
template <int ROWB>
__device__ static inline int v_swz(int row) {
  static_assert(ROWB == 128 || ROWB == 256, "V tile rows of 64 or 128 bf16");
  return ROWB == 128 ? 2 * (row & 3) + ((row >> 2) & 1) : 4 * (row & 3);
}

// Direct global -> LDS load of 16 bytes per lane (global_load_lds_dwordx4): lane i of the wave
// writes the 16 bytes at gsrc (its own address) to LDS at lds_wave_base + 16 i.  The load is
// counted by vmcnt like any global load, but it is issued from inline assembly so that the
// compiler does not serialise later LDS reads behind it: the caller waits (wait_vmcnt0) and
// synchronises before anyone reads the destination.
__device__ static inline void dma16_to_lds(const void* gsrc, void* lds_wave_base) {
  const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(base) : "memory", "m0");
}
__device__ static inline void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only

// Workgroup barrier that orders LDS traffic only: __syncthreads() also waits for every global load and
// store in flight, which would expose the latency of the next tile's prefetch and of the output stores at
// each of a tile's barriers.  Registers filled by global loads are private to the lane; the compiler
// still waits for them where they are used.  Not for data that reaches LDS by direct global -> LDS loads:
// those need wait_vmcnt0() before the barrier.
__device__ static inline void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Raises a kernel's dynamic-LDS limit when it needs more than the default; done once per kernel
// and size (the attribute call is host work we do not want on every launch).
template <typename KernelT>
static dark_status allow_lds(KernelT kernel, size_t bytes) {
  if (bytes > 160 * 1024) return DARK_EUNSUPPORTED;
  if (bytes <= 48 * 1024) return DARK_OK;
  static size_t granted = 0;  // one instance per kernel type
  static const void* granted_for = nullptr;
  const void* fn = reinterpret_cast<const void*>(kernel);
  if (granted_for == fn && granted >= bytes) return DARK_OK;
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return DARK_EHIP;
  granted = bytes;
  granted_for = fn;
  return DARK_OK;
}

}  // namespace fz

// Slicing of a sequence for the causal kernels: about one workgroup per CU over all (b,h), slices of whole
// 64-token tiles, at most 64 per (b,h).  Forward and backward must agree on it.
inline void causal_slices(const Problem& pb, int* P, int* slice_len) {
  const dark_params& p = pb.p;
  long long want = (p.sched_cs_wgs > 0 ? p.sched_cs_wgs : 256) / (pb.BH() > 0 ? pb.BH() : 1);
  want = want < 1 ? 1 : (want > 64 ? 64 : want);
  int sl = (int)((p.L + want - 1) / want);
  sl = ((sl + 63) / 64) * 64;
  if (sl < 64) sl = 64;
  *slice_len = sl;
  *P = p.L > 0 ? (p.L + sl - 1) / sl : 1;
}
// What the causal forward can hand to the backward (and what both otherwise keep in the workspace): the fp16
// operand copies, the key norms and the exclusive prefix states with their running shifts.
struct CausalKeep {
  _Float16 *Ah, *Mh;
  float *Spre, *zpre, *cpre, *nrm;
};
inline CausalKeep take_causal_keep(Arena& a, const Problem& pb, int P) {
  const dark_params& p = pb.p;
  const size_t nstate = (size_t)pb.BH() * P * p.m;
  CausalKeep k;
  k.Ah = a.take<_Float16>((size_t)p.H * p.m * p.d);
  k.Mh = a.take<_Float16>((size_t)p.H * p.r * p.d);
  k.Spre = a.take<float>(nstate * p.dv);
  k.zpre = a.take<float>(nstate);
  k.cpre = a.take<float>((size_t)pb.BH() * P);
  k.nrm = a.take<float>((size_t)pb.BH() * (p.L > 0 ? p.L : 1));
  return k;
}

// Implemented in fused.hip, used by the other fused translation units as well.
// A' = sqrt(scale) log2(e) W M as fp16 [H][m][d];  M' = sqrt(scale) sqrt(log2(e)/2) M as fp16 [H][r][d].
// Requires r, d multiples of 4, d <= 256, r * d <= 16384.
dark_status fused_launch_prep(const Problem& pb, const float* M, const float* W, _Float16* Ah, _Float16* Mh);
// Key/value pass over P slices of slice_len tokens (a multiple of 64) per (b,h):
// Spart [BH][P][m][dv] (bf16), zpart and cpart [BH][P][m] (per-slice, per-feature shifts, log2 domain).
// nrm_out (may be null): [BH][L], receives the key norms |M' k|^2 that the pass computes on its way.
// Requires d = r = dv = 64.
dark_status fused_launch_kv_reduce(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                   const _Float16* Mh, unsigned short* Spart, float* zpart, float* cpart, int P,
                                   int slice_len, float* nrm_out = nullptr);
// Implemented in fused_scan.hip: the scan over the tiles of every slice, from the prefix states.
dark_status fused_launch_scan_ws(const Problem& pb, const void* Q, const void* K, const void* V, const _Float16* Ah,
                                 const float* nrm, const float* Spre, const float* zpre, const float* cpre, void* out,
                                 int P, int slice_len);
// Implemented in fused_causal.hip.
bool fused_causal_supported(const Problem& pb);
// Key norms nrm [BH][L], slice states ([BH][P][m][dv] bf16 with per-feature shifts) and their exclusive prefix
// Spre, zpre (fp32, expressed in the running scalar shift cpre [BH][P]) for d = r = dv = 64.
dark_status fused_causal_states64(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                  const _Float16* Mh, float* nrm, unsigned short* Spart, float* zpart, float* cpart,
                                  float* Spre, float* zpre, float* cpre, int P, int slice_len);
// The same states for d = r = dv = 128 (whose accumulators do not fit k_kv_reduce's register budget):
// key norms into nrm [BH][L], then an 8-wave kernel per (b,h, slice).
dark_status fused_launch_slice_state128(const Problem& pb, const void* K, const void* V, const _Float16* Ah,
                                        const _Float16* Mh, float* nrm, unsigned short* Spart, float* zpart,
                                        float* cpart, int P, int slice_len);

}  // namespace dark

// Device-side helpers shared by the Sparrow HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sparrow {

typedef unsigned short bf16_t;  // raw bfloat16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Finite stand-in for "no score seen yet": exp2(kNegBig - x) underflows to 0 for any real x and
// kNegBig - kNegBig = 0 never produces a NaN.
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((unsigned int)b) << 16);
}
// Two packed bf16 (low half = element 0) -> floats.
__device__ __forceinline__ float bf16lo_to_f32(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(unsigned int w) {
  return __uint_as_float(w & 0xffff0000u);
}
// Round to nearest even; inputs are finite or +-inf (NaN is passed through as a quiet NaN).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// Two floats -> packed bf16 (low half = lo) with the hardware conversion (v_cvt_pk_bf16_f32,
// round to nearest even).
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(unsigned int, v);
}

// fp16 pairs (round to nearest even) and back.
__device__ __forceinline__ unsigned int pack_f16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
  const f16x2 v = {(_Float16)lo, (_Float16)hi};
  return __builtin_bit_cast(unsigned int, v);
}
__device__ __forceinline__ f32x4 unpack_f16x4(unsigned int w0, unsigned int w1) {
  typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
  const f16x2 a = __builtin_bit_cast(f16x2, w0), b = __builtin_bit_cast(f16x2, w1);
  return (f32x4){(float)a[0], (float)a[1], (float)b[0], (float)b[1]};
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Element type traits for kernels templated on the storage type.
template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPer16B = 4;
  static __device__ __forceinline__ void unpack(const u32x4 &w, float *f) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;
  static __device__ __forceinline__ void unpack(const u32x4 &w, float *f) {
    f[0] = bf16lo_to_f32(w.x); f[1] = bf16hi_to_f32(w.x);
    f[2] = bf16lo_to_f32(w.y); f[3] = bf16hi_to_f32(w.y);
    f[4] = bf16lo_to_f32(w.z); f[5] = bf16hi_to_f32(w.z);
    f[6] = bf16lo_to_f32(w.w); f[7] = bf16hi_to_f32(w.w);
  }
  static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// Butterfly reductions over a 64-lane wavefront (all lanes get the result).
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Cross-lane helpers on the vector ALU (DPP and the gfx950 row-swap instructions) instead of
// ds_bpermute, which goes through the LDS crossbar.
template <int kCtrl> __device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kCtrl, 0xF, 0xF, true));
}
// Sum over aligned groups of N consecutive lanes (N = 8, 16 or 32); every lane gets the result.
template <int N> __device__ __forceinline__ float group_sum(float v) {
  static_assert(N == 8 || N == 16 || N == 32, "lane group size");
  v += dpp_f32<0xB1>(v);          // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);          // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);         // row_half_mirror: lanes i <-> 7-i of each 8
  if (N >= 16) v += dpp_f32<0x140>(v);   // row_mirror: lanes i <-> 15-i of each 16
  if (N >= 32) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  return v;
}
// Sum over the whole wavefront on the vector ALU (every lane gets the result).
__device__ __forceinline__ float wave_sum_valu(float v) {
  v = group_sum<32>(v);
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Maximum (float) / minimum (int) over the whole wavefront on the vector ALU; every lane gets it.
__device__ __forceinline__ float wave_max_valu(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  v = fmaxf(v, dpp_f32<0x140>(v));
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
template <int kCtrl> __device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xF, 0xF, true);
}
__device__ __forceinline__ int wave_min_valu(int v) {
  v = min(v, dpp_i32<0xB1>(v));
  v = min(v, dpp_i32<0x4E>(v));
  v = min(v, dpp_i32<0x141>(v));
  v = min(v, dpp_i32<0x140>(v));
  auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
  v = min((int)r[0], (int)r[1]);
  r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
  return min((int)r[0], (int)r[1]);
}
// Value of lane (lane ^ O) for O = 8, 16 or 32.
template <int O> __device__ __forceinline__ float lane_xor(float v, int lane) {
  static_assert(O == 8 || O == 16 || O == 32, "supported distances");
  if (O == 8) return dpp_f32<0x128>(v);              // row_ror 8 within each row of 16
  if (O == 16) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((lane & 16) ? r[0] : r[1]);
  }
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float((lane & 32) ? r[0] : r[1]);
}

// Ancestor-or-self bit set of draft row i: bit j set <=> row i may attend draft row j.
// parent == nullptr means a chain.  Requires parent[a] < a (then the walk ends) and i < 64.
__device__ __forceinline__ unsigned long long ancestor_mask(const int32_t *parent, int i) {
  if (parent == nullptr) return (2ull << i) - 1ull;
  unsigned long long m = 0;
  int a = i;
  // At most i+1 steps: a strictly decreases for a valid tree; the counter bounds the walk for
  // an invalid one.
  for (int steps = 0; a >= 0 && steps <= i; ++steps) {
    m |= 1ull << a;
    int p = parent[a];
    a = (p < a) ? p : -1;
  }
  return m;
}

// Same bit set, computed by a whole wavefront at once: lane j keeps parent[j] in a register and
// every lane walks its own row's path with cross-lane reads, so the walk costs one global load
// instead of one per tree level.  Must be called by all 64 lanes (i may differ per lane);
// n_q <= 64.
__device__ __forceinline__ unsigned long long ancestor_mask_wave(const int32_t *parent, int n_q,
                                                                 int i, int lane) {
  if (parent == nullptr) return (2ull << i) - 1ull;
  const int pv = lane < n_q ? parent[lane] : -1;
  unsigned long long m = 0;
  int a = i;
  for (int steps = 0; steps < n_q && __builtin_amdgcn_ballot_w64(a >= 0) != 0ull; ++steps) {
    if (a >= 0) m |= 1ull << a;
    const int p = __shfl(pv, a >= 0 ? a : 0, 64);
    a = (a >= 0 && p < a) ? p : -1;
  }
  return m;
}

}  // namespace sparrow

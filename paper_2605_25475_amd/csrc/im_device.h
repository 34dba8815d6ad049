// Device-side helpers shared by the kernels of libindexmem (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;

#define IM_D 128      // head_dim
#define IM_DI 64      // idx_dim (state per KV head)
#define IM_DI_SHARED 16   // idx_dim of the head-shared layout (d_head / 8: Section 4, hyper-parameters)
#define IM_DM 128     // mem_dim
#define IM_WAVE 64

// bits of the device-side status word (the public header names them without the suffix)
#define IM_STATUS_APPEND_OVERFLOW_BIT 1
#define IM_STATUS_LIVE_EXCEEDED_BIT 2
#define IM_STATUS_OVER_BUDGET_BIT 8

__device__ __forceinline__ float bf2f(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even
__device__ __forceinline__ bf16_t f2bf_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// fp64 -> bf16 with ONE rounding (nearest even): truncate to fp32 with a sticky last bit
// (round to odd), which is innocuous because fp32 carries 16 more bits than bf16, then round.
__device__ __forceinline__ bf16_t d2bf_rne(double x) {
  float f = __double2float_rz(x);
  uint32_t u = __float_as_uint(f);
  if ((double)f != x) u |= 1u;
  return f2bf_rne(__uint_as_float(u));
}

// order-preserving map of a score to an unsigned key (larger score <-> larger key); -0 == +0
__device__ __forceinline__ uint32_t score_key(float s) {
  if (s == 0.0f) s = 0.0f;
  uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
#define IM_KEY_PINF 0xff800000u  // score_key(+inf)

// ---- wave64 reductions on the VALU's DPP paths (ds_bpermute-based shuffles are far slower here) ----
// row_shr:n = 0x110 + n, row_bcast:15 = 0x142, row_bcast:31 = 0x143.  After the six steps lane 63
// holds the reduction of all 64 lanes; it is returned as a wave-uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_zero_f(float v) {   // lanes without a source read 0
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, true));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_keep_f(float v) {   // lanes without a source read their own value
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_f(float v) {
  v += dpp_zero_f<0x111, 0xF>(v);
  v += dpp_zero_f<0x112, 0xF>(v);
  v += dpp_zero_f<0x114, 0xF>(v);
  v += dpp_zero_f<0x118, 0xF>(v);
  v += dpp_zero_f<0x142, 0xA>(v);
  v += dpp_zero_f<0x143, 0xC>(v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_f(float v) {
  v = fmaxf(v, dpp_keep_f<0x111, 0xF>(v));
  v = fmaxf(v, dpp_keep_f<0x112, 0xF>(v));
  v = fmaxf(v, dpp_keep_f<0x114, 0xF>(v));
  v = fmaxf(v, dpp_keep_f<0x118, 0xF>(v));
  v = fmaxf(v, dpp_keep_f<0x142, 0xA>(v));
  v = fmaxf(v, dpp_keep_f<0x143, 0xC>(v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_keep_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_min_u(uint32_t v) {
  v = min(v, dpp_keep_u<0x111, 0xF>(v));
  v = min(v, dpp_keep_u<0x112, 0xF>(v));
  v = min(v, dpp_keep_u<0x114, 0xF>(v));
  v = min(v, dpp_keep_u<0x118, 0xF>(v));
  v = min(v, dpp_keep_u<0x142, 0xA>(v));
  v = min(v, dpp_keep_u<0x143, 0xC>(v));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t wave_max_u(uint32_t v) {
  v = max(v, dpp_keep_u<0x111, 0xF>(v));
  v = max(v, dpp_keep_u<0x112, 0xF>(v));
  v = max(v, dpp_keep_u<0x114, 0xF>(v));
  v = max(v, dpp_keep_u<0x118, 0xF>(v));
  v = max(v, dpp_keep_u<0x142, 0xA>(v));
  v = max(v, dpp_keep_u<0x143, 0xC>(v));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_zero_d(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, ROW_MASK, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROW_MASK, 0xF, true);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double wave_sum_d(double v) {
  v += dpp_zero_d<0x111, 0xF>(v);
  v += dpp_zero_d<0x112, 0xF>(v);
  v += dpp_zero_d<0x114, 0xF>(v);
  v += dpp_zero_d<0x118, 0xF>(v);
  v += dpp_zero_d<0x142, 0xA>(v);
  v += dpp_zero_d<0x143, 0xC>(v);
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), 63);
  const int hi = __builtin_amdgcn_readlane((int)(b >> 32), 63);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// sum over the 4 lanes l, l^16, l^32, l^48 (the same position in the four 16-lane rows), returned
// in every lane: two swaps of 16- and 32-lane halves (gfx950 v_permlane16_swap / v_permlane32_swap)
__device__ __forceinline__ float rows_sum_f(float v) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float rows_max_f(float v) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ double rows_sum_d(double v) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  unsigned int lo = (unsigned int)b, hi = (unsigned int)(b >> 32);
  u2 rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
  u2 rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
  double s = __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
             __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
  const unsigned long long c = (unsigned long long)__double_as_longlong(s);
  lo = (unsigned int)c; hi = (unsigned int)(c >> 32);
  rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
  rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
  return __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
         __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
}
// Wave sums of NV (8 or 16) doubles at once, as a butterfly: a swap of 32-lane halves folds two values
// into one register (value 2 i in the lower half, value 2 i + 1 in the upper), a swap of 16-lane rows
// folds two of those (one value per row), and only the last step, the sum over the 16 lanes of a row,
// is done per register: 42 instructions for 8 values where 8 separate wave sums take 160.
// On return lane 15 of row rho (lane 16 rho + 15) of s[i] holds the wave's sum of value
// 4 i + 2 (rho & 1) + (rho >> 1).
template <int NV>
__device__ __forceinline__ void wave_sums_butterfly_d(const double* v, double* s) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  auto lo = [](double x) { return (unsigned int)(unsigned long long)__double_as_longlong(x); };
  auto hi = [](double x) { return (unsigned int)((unsigned long long)__double_as_longlong(x) >> 32); };
  auto mk = [](unsigned int l, unsigned int h) { return __longlong_as_double((long long)(((unsigned long long)h << 32) | l)); };
  double r[NV / 2];
#pragma unroll
  for (int i = 0; i < NV / 2; ++i) {
    const u2 pl = __builtin_amdgcn_permlane32_swap(lo(v[2 * i]), lo(v[2 * i + 1]), false, false);
    const u2 ph = __builtin_amdgcn_permlane32_swap(hi(v[2 * i]), hi(v[2 * i + 1]), false, false);
    r[i] = mk(pl[0], ph[0]) + mk(pl[1], ph[1]);
  }
#pragma unroll
  for (int i = 0; i < NV / 4; ++i) {
    const u2 pl = __builtin_amdgcn_permlane16_swap(lo(r[2 * i]), lo(r[2 * i + 1]), false, false);
    const u2 ph = __builtin_amdgcn_permlane16_swap(hi(r[2 * i]), hi(r[2 * i + 1]), false, false);
    double t = mk(pl[0], ph[0]) + mk(pl[1], ph[1]);
    t += dpp_zero_d<0x111, 0xF>(t);   // row_shr 1, 2, 4, 8: lane 15 of each row ends with the row's sum
    t += dpp_zero_d<0x112, 0xF>(t);
    t += dpp_zero_d<0x114, 0xF>(t);
    t += dpp_zero_d<0x118, 0xF>(t);
    s[i] = t;
  }
}

// v + (the same lane of the other 32-lane half), in every lane
__device__ __forceinline__ float halves_sum_f(float v) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// a 16-byte load with the streaming hint: data that is read once per step
typedef unsigned int dec_u4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const dec_u4 v = __builtin_nontemporal_load((const dec_u4*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

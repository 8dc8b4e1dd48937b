// Device helpers for the gfx950 kernels: wave64 DPP reductions, typed 16-byte
// loads, bf16 dot products, block scans.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sagekv {

constexpr int kWave = 64;

enum : int { DT_BF16 = 0, DT_F32 = 1 };

// ---- element traits --------------------------------------------------------------------
template <int DT>
struct Elem;
template <>
struct Elem<DT_BF16> {
  static constexpr int bytes = 2;
  static constexpr int per_lane = 8;  // elements in one 16-byte load
};
template <>
struct Elem<DT_F32> {
  static constexpr int bytes = 4;
  static constexpr int per_lane = 4;
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// 16 bytes of K (or V) against 16 bytes of q, accumulated in fp32.
template <int DT>
__device__ __forceinline__ float dot16(const uint4& a, const uint4& b, float acc);

template <>
__device__ __forceinline__ float dot16<DT_BF16>(const uint4& a, const uint4& b, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
  return acc;
}
template <>
__device__ __forceinline__ float dot16<DT_F32>(const uint4& a, const uint4& b, float acc) {
  acc = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc);
  acc = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc);
  acc = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc);
  acc = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc);
  return acc;
}

// The 16 bytes of one lane as fp32 values (8 for bf16, 4 for fp32).
template <int DT>
__device__ __forceinline__ void unpack16(const uint4& a, float* f);
template <>
__device__ __forceinline__ void unpack16<DT_BF16>(const uint4& a, float* f) {
  f[0] = bf16_lo(a.x); f[1] = bf16_hi(a.x); f[2] = bf16_lo(a.y); f[3] = bf16_hi(a.y);
  f[4] = bf16_lo(a.z); f[5] = bf16_hi(a.z); f[6] = bf16_lo(a.w); f[7] = bf16_hi(a.w);
}
template <>
__device__ __forceinline__ void unpack16<DT_F32>(const uint4& a, float* f) {
  f[0] = __uint_as_float(a.x); f[1] = __uint_as_float(a.y); f[2] = __uint_as_float(a.z); f[3] = __uint_as_float(a.w);
}

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// Streaming 16-byte load (data read once: do not keep it in the caches).
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16(void* p, const uint4& v) { *reinterpret_cast<uint4*>(p) = v; }

// ---- cross-lane sums -----------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Sum over aligned groups of LANES consecutive lanes; every lane of the group gets the total.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 1 || LANES == 2 || LANES == 4 || LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "");
  if (LANES >= 2) v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
  if (LANES >= 4) v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
  if (LANES >= 8) v += dpp_f32<0x141>(v);  // row_half_mirror
  if (LANES >= 16) v += dpp_f32<0x140>(v); // row_mirror
  if (LANES >= 32) v += __shfl_xor(v, 16);
  if (LANES >= 64) v += __shfl_xor(v, 32);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// exp(x) * inv for x <= 0-ish and a normal `inv` in [2^-62, 1] (a softmax weight: inv = 1/Z), via the
// hardware exp2 with the rounding error of x*log2(e) folded back in (relative error a few 1e-7 where
// the result is a normal number).  The hardware exp2 returns 0 for every result under 2^-126, whereas
// the product is wanted correctly rounded all the way down through the denormal range (scores are
// RANKED, and fp32 keeps denormals): an argument more than 64 octaves down is raised by 64 octaves
// before exp2 (exact: the sum has a finer ulp than the argument) and the factor is lowered by 2^-64
// instead, so the final multiply rounds into the denormal range like any fp32 product.  Results
// under 2^-190 * inv come out as 0, which is also their nearest fp32 value.
__device__ __forceinline__ float exp_times(float x, float inv) {
  const float l2e_hi = 1.44269502162933349609375f;  // float(log2 e)
  const float l2e_lo = 1.92596299112661746e-8f;     // log2 e - l2e_hi
  const float t = x * l2e_hi;
  float e = fmaf(x, l2e_hi, -t);
  e = fmaf(x, l2e_lo, e);
  const bool far = t < -64.f;
  float r = __builtin_amdgcn_exp2f(far ? t + 64.f : t);
  r = fmaf(r, e * 0.693147182464599609375f, r);
  return r * (far ? inv * 0x1p-64f : inv);
}

// Absolute slack that goes with the relative band around a coarse k-th score: below 2^-126 an fp32
// score is a multiple of 2^-149, each head's term is rounded to that grid, and up to 64 heads add up.
constexpr float kDenormSlack = 0x1p-142f;

__device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.44269502162933349609375f); }

// Which terms of a head's softmax sum need an fp64 exponent.  An fp32 logit of magnitude |l| carries an
// absolute error of about eps = 1.2e-7 |l| (rms, measured: a head with 40-95 % of its mass on one token
// of logit 36 had its Z off by 2-3e-6), its exponential the same relative error.  Terms of weight w_i
// (share of Z) with independent errors put Z off by eps * sqrt(sum w_i^2) <= eps * sqrt(theta) if every
// term of weight >= theta is exact; theta = (1e-7 / eps)^2 keeps that at 1e-7, a third of what could
// move two group-sum scores past the 1e-6 that a kept set may differ by.  M, Z: the head's (estimated)
// maximum logit and sum of exp(l - M); returns the logit whose term has weight theta (+inf: no term
// qualifies).  The terms above it are few by construction: at most 1 / theta = 1.4 M^2 per head.
__host__ __device__ inline float heavy_logit_threshold(float M, float Z) {
  if (!(Z > 0.f) || !(M == M)) return INFINITY;
  const float mag = fabsf(M) > 4.f ? fabsf(M) : 4.f;
  const float r = 1e-7f / (1.2e-7f * mag);
  return M + logf(r * r * Z);
}

// ---- block-wide inclusive scan of one int per thread (blockDim.x = NT, multiple of 64) ---------
// `wave_tot` is NT/64 ints of shared memory.  Returns the inclusive prefix; *total gets the block sum.
template <int NT>
__device__ __forceinline__ int block_scan_incl(int v, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_up(x, o);
    if (lane >= o) x += y;
  }
  __syncthreads();  // protects wave_tot against the previous use
  if (lane == 63) wave_tot[w] = x;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) {
    int t = wave_tot[i];
    if (i < w) base += t;
    tot += t;
  }
  *total = tot;
  return x + base;
}

}  // namespace sagekv

// Shared device helpers for the gfx950 ERNIE kernels: vector types, MFMA
// fragment conventions and wave64 reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace ernie {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kHeadDim = 64;

// v_mfma_f32_32x32x16_f16 operand convention used everywhere in this library
// (one wave64 computes D[32x32] += A[32x16] * B[16x32]):
//   A fragment: lane l holds A[l % 32][8 * (l / 32) + 0..7]
//   B fragment: lane l holds B[8 * (l / 32) + 0..7][l % 32]
//   D fragment: lane l, register v (0..15) holds D[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
// Both inputs are therefore "8 consecutive k per lane, lane % 32 selects the
// row / column", which is what a K-contiguous (row-major [rows, K]) operand
// delivers with one 16-byte load per lane.
__device__ __forceinline__ floatx16 mfma32(half8 a, half8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int mfma32_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Packed weight layout ("fragment-major"): a [N, K] row-major matrix becomes
// tiles of 32 rows x 16 k, each stored as the 64 lanes' 8-half fragments in
// lane order (1 KiB, contiguous), tiles ordered [n_tile][k_tile].  A wave reads
// one operand fragment with a single fully coalesced 16-byte-per-lane load.
__host__ __device__ __forceinline__ size_t packed_frag_offset(int n_tile, int k_tile, int k_tiles) {
  return ((size_t)n_tile * k_tiles + k_tile) * 512;   // in halves
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// (value, index) maximum with the lowest index winning exact ties.
__device__ __forceinline__ void argmax_merge(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// erf by the rational-exponential formula 7.1.26 of Abramowitz & Stegun,
//   erf(x) = 1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),  x >= 0,
// branch-free (about a dozen instructions against the several ranges of the library routine).  In fp32 it
// is within 6.1e-7 of erf over the whole line, so the erf-form GELU below is within 4.7e-7 absolute of the
// exact one: three orders of magnitude below the fp16 rounding of its result.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(1.0f + 0.3275911f * ax);
  const float poly = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
  return copysignf(1.0f - poly * __expf(-ax * ax), x);
}

// The erf-form GELU twice: with the library erf (cheapest where the epilogue is throughput-bound, as in the
// prefill GEMM: most arguments take its short polynomial range) and with the branch-free formula (cheapest
// where a few waves wait on the epilogue's latency, as in the decode-step kernels).
__device__ __forceinline__ float gelu_erf(float a) {
  return a * 0.5f * (1.0f + erff(a * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_erf_fast(float a) {
  return a * 0.5f * (1.0f + erf_as(a * 0.70710678118654752440f));
}

// Workgroup id -> logical id such that the workgroups of one XCD (ids congruent mod 8) cover a
// contiguous range of logical ids: neighbours in the logical order then share that XCD's L2.
__device__ __forceinline__ int xcd_contiguous_id(int id, int total) {
  const int x = id & 7, q = total >> 3, r = total & 7;
  return x * q + min(x, r) + (id >> 3);
}

}  // namespace ernie

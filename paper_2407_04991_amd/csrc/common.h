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

// Warm-up of what the NEXT kernel of the decode step will read first.  The decode GEMMs on fp16 activations
// are short and leave most compute units idle; a few extra workgroups appended to such a launch pull the
// packed weight matrix of the LayerNorm-prologue GEMM that follows into the L2 of the XCD whose workgroups
// will read it (workgroup ids congruent mod 8 run on one XCD, and that consumer orders its ids
// XCD-contiguously), plus the small vectors every consumer workgroup starts with, so that the consumer's
// memory round trip ends in that L2 instead of in HBM.  The loaded values are discarded; a wrong guess of
// the mapping costs time, never correctness.
struct DecPrefetch {
  const unsigned char* ptr;   // packed weight matrix (fragment-major strips); null = nothing to do
  unsigned strip_bytes;       // bytes of one 32-column strip (K * 64), a multiple of 16
  int n_strips;
  // the consumer's grid: `cons_grid` workgroups in XCD-contiguous order, `cons_zg` row groups per strip group,
  // `cons_ns` strips per group
  int cons_grid, cons_zg, cons_ns;
  int count;                  // warming workgroups (a multiple of 8)
  // small per-layer vectors (biases, LayerNorm scale / shift) that EVERY workgroup of the consumer, or of the
  // kernel after it, reads first: each XCD's warming workgroups load all of them (multiples of 16 bytes; null = none)
  const unsigned char* aux[2];
  unsigned aux_bytes[2];
};

// idx = rank among the warming workgroups, wg_id = the workgroup's linear id in its grid (its XCD is wg_id % 8);
// ranks 8 j .. 8 j + 7 must sit on 8 different XCDs (consecutive linear ids)
__device__ __forceinline__ void dec_prefetch_run(const DecPrefetch& f, int idx, int wg_id, int tid, int nthreads) {
  const int x = wg_id & 7, j = idx >> 3, per = f.count >> 3;
  if (per <= 0) return;
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    if (!f.aux[a]) continue;
    const unsigned n16 = f.aux_bytes[a] >> 4;
    for (unsigned u = (unsigned)j * nthreads + tid; u < n16; u += (unsigned)per * nthreads) {
      const uint4 v = *reinterpret_cast<const uint4*>(f.aux[a] + (size_t)u * 16);
      asm volatile("" ::"v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w));
    }
  }
  if (!f.ptr) return;
  // XCD x runs the consumer's logical ids [lo, lo + cnt), i.e. a contiguous range of strips
  const int q = f.cons_grid >> 3, r = f.cons_grid & 7;
  const int lo = x * q + min(x, r), cnt = q + (x < r ? 1 : 0);
  if (cnt <= 0) return;
  const int s_lo = (lo / f.cons_zg) * f.cons_ns;
  const int s_n = min(((lo + cnt - 1) / f.cons_zg + 1) * f.cons_ns, f.n_strips) - s_lo;
  if (s_n <= 0) return;
  const unsigned upb = f.strip_bytes >> 4;                       // 16-byte units per strip
  const unsigned units = (unsigned)s_n * upb;
  const unsigned u0 = (unsigned)((unsigned long long)units * j / per), u1 = (unsigned)((unsigned long long)units * (j + 1) / per);
  constexpr int kFlight = 8;
  const unsigned char* base = f.ptr + (size_t)s_lo * f.strip_bytes;      // the XCD's strips are contiguous bytes
  for (unsigned u = u0 + tid; u < u1; u += nthreads * kFlight) {
    uint4 v[kFlight];
#pragma unroll
    for (int k = 0; k < kFlight; ++k)      // clamped, not predicated: all loads issue together
      v[k] = *reinterpret_cast<const uint4*>(base + (size_t)min(u + k * nthreads, u1 - 1) * 16);
#pragma unroll
    for (int k = 0; k < kFlight; ++k) asm volatile("" ::"v"(v[k].x), "v"(v[k].y), "v"(v[k].z), "v"(v[k].w));
  }
}

// Warm-up of the key/value cache rows the next decode attention will stream: the attention workgroup of
// (head h, batch row b) has id h + H b, so XCD x reads the streams with (h + H b) % 8 == x.
struct KvPrefetch {
  const unsigned char* k;     // layer bases of the K and V caches [Bmax][H][S][64] fp16; null = nothing to do
  const unsigned char* v;
  const int* slot;            // cache row of batch row b, or null
  int B, H, S, rows;          // rows = upper bound of the valid rows of any stream (<= S)
  int count;                  // warming workgroups (a multiple of 8)
};

__device__ __forceinline__ void kv_prefetch_run(const KvPrefetch& f, int idx, int wg_id, int tid, int nthreads) {
  if (!f.k) return;
  const int x = wg_id & 7, j = idx >> 3, per = f.count >> 3;
  if (per <= 0) return;
  const int n_streams = f.B * f.H;
  // every stream is fetched up to the longest one's length: reading the per-row lengths first would put a
  // second memory round trip in front of the fetch, which then outlasts the host kernel (measured: a loss)
  const unsigned units = (unsigned)f.rows * 8;                   // 16-byte units per stream and tensor
  for (int s = x + 8 * j; s < n_streams; s += 8 * per) {
    const int b = s / f.H, h = s - b * f.H;
    const int cb = f.slot ? f.slot[b] : b;
    const size_t base = ((size_t)cb * f.H + h) * f.S * 128;
    for (unsigned u = tid; u < units; u += nthreads * 4) {
      floatx4 kk[4], vv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {      // clamped, not predicated: all loads issue together
        const size_t off = base + (size_t)min(u + q * nthreads, units - 1) * 16;
        kk[q] = *reinterpret_cast<const floatx4*>(f.k + off);
        vv[q] = *reinterpret_cast<const floatx4*>(f.v + off);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        asm volatile("" ::"v"(kk[q][0]), "v"(kk[q][1]), "v"(kk[q][2]), "v"(kk[q][3]));
        asm volatile("" ::"v"(vv[q][0]), "v"(vv[q][1]), "v"(vv[q][2]), "v"(vv[q][3]));
      }
    }
  }
}

}  // namespace ernie

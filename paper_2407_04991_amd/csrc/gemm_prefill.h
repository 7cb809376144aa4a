// Epilogues of the prefill GEMMs (the kernel itself is in gemm_prefill2.h).
// The kernel transposes each finished 32 x 32 accumulator tile through LDS and
// calls store8(row, col, v) once per run of 8 consecutive columns of one row
// (col % 8 == 0, col + 8 <= N, v = accumulator + bias in fp32), so that every
// epilogue writes 16-byte (fp16) or 32-byte (fp32) pieces.
#pragma once

#include "common.h"

namespace ernie {

__device__ __forceinline__ half8 to_half8(const float (&v)[8]) {
  half8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (half_t)v[j];
  return o;
}

// QKV projection: scatter Q to [H][T][64] and K, V straight into the
// head-major cache [B][H][S][64] of this layer (8 consecutive columns stay inside one head).
struct EpiQKV {
  half_t* q;            // [H][T][64]
  half_t* kcache;       // layer base of K: [Bmax][H][S][64]
  half_t* vcache;
  const int* tok_seq;   // [T]
  const int* tok_pos;   // [T]
  int d, H, S, T;
  __device__ __forceinline__ void store8(int row, int col, const float (&v)[8]) const {
    const int part = col / d, within = col - part * d;
    const int head = within >> 6, e = within & 63;
    half_t* dst;
    if (part == 0) {
      dst = q + ((size_t)head * T + row) * 64 + e;
    } else {
      const int b = tok_seq[row], pos = tok_pos[row];
      dst = ((part == 1) ? kcache : vcache) + (((size_t)b * H + head) * S + pos) * 64 + e;
    }
    *reinterpret_cast<half8*>(dst) = to_half8(v);
  }
};

// out-projection / FFN2: Y = acc + bias + residual, fp16 (LayerNorm follows in its own pass).
struct EpiResidual {
  const half_t* res;   // [M, N]
  half_t* y;           // [M, N]
  int N;
  __device__ __forceinline__ half8 load8(int row, int col) const {
    return *reinterpret_cast<const half8*>(res + (size_t)row * N + col);
  }
  __device__ __forceinline__ void store8(int row, int col, const float (&v)[8], half8 r) const {
    half8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = (half_t)(v[j] + (float)r[j]);
    *reinterpret_cast<half8*>(y + (size_t)row * N + col) = out;
  }
};

// FFN1: G = gelu(acc + bias), fp16.  FAST picks the branch-free erf (decode step) over the library one (prefill).
template <bool FAST>
struct EpiGeluT {
  half_t* g;
  int N;
  __device__ __forceinline__ void store8(int row, int col, const float (&v)[8]) const {
    half8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = (half_t)(FAST ? gelu_erf_fast(v[j]) : gelu_erf(v[j]));
    *reinterpret_cast<half8*>(g + (size_t)row * N + col) = out;
  }
};
using EpiGelu = EpiGeluT<false>;
using EpiGeluFast = EpiGeluT<true>;

// Raw fp32 output [gridDim.y][M, N]: one partial buffer per split of the contraction (decode step at
// large batch: the consumer kernels add the partials, bias and residual).
struct EpiRaw32 {
  float* r;
  int N;
  size_t slab;   // M * N
  __device__ __forceinline__ void store8(int row, int col, const float (&v)[8]) const {
    float* dst = r + blockIdx.y * slab + (size_t)row * N + col;
    *reinterpret_cast<float4*>(dst) = float4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4*>(dst + 4) = float4{v[4], v[5], v[6], v[7]};
  }
};

}  // namespace ernie

// Epilogues of the prefill GEMMs (the kernel itself is in gemm_prefill2.h).
// An epilogue is called once per finished accumulator element with
// (row, col, value including bias).
#pragma once

#include "common.h"

namespace ernie {

// QKV projection: scatter Q to [H][T][64] and K, V straight into the
// head-major cache [B][H][S][64] of this layer.
struct EpiQKV {
  half_t* q;            // [H][T][64]
  half_t* kcache;       // layer base of K: [Bmax][H][S][64]
  half_t* vcache;
  const int* tok_seq;   // [T]
  const int* tok_pos;   // [T]
  int d, H, S, T;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    const int part = col / d, within = col - part * d;
    const int head = within >> 6, e = within & 63;
    if (part == 0) {
      q[((size_t)head * T + row) * 64 + e] = (half_t)v;
    } else {
      const int b = tok_seq[row], pos = tok_pos[row];
      half_t* base = (part == 1) ? kcache : vcache;
      base[(((size_t)b * H + head) * S + pos) * 64 + e] = (half_t)v;
    }
  }
};

// out-projection / FFN2: Y = acc + bias + residual, fp16 (LayerNorm follows in its own pass).
struct EpiResidual {
  const half_t* res;   // [M, N]
  half_t* y;           // [M, N]
  int N;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    const size_t o = (size_t)row * N + col;
    y[o] = (half_t)(v + (float)res[o]);
  }
};

// FFN1: G = gelu(acc + bias), fp16.
struct EpiGelu {
  half_t* g;
  int N;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    g[(size_t)row * N + col] = (half_t)gelu_erf(v);
  }
};

// Raw fp32 output [M, N] (decode step at large batch: the consumer kernels add bias and residual).
struct EpiRaw32 {
  float* r;
  int N;
  __device__ __forceinline__ void operator()(int row, int col, float v) const { r[(size_t)row * N + col] = v; }
};

}  // namespace ernie

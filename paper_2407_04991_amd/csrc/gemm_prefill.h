// Prefill GEMM on FP16 MFMA: C[M, N] = A[M, K] * W[N, K]^T with fused epilogues.
//
// A is row-major fp16 (packed prompt tokens), W is the fragment-major packed
// weight.  One workgroup of 256 threads (2 x 2 waves) owns a 128 x 128 output
// tile and walks K in steps of 64 through double-buffered LDS:
//   A tile  128 rows x 64 k, row-major with an 8-half pad per row (144-byte
//           pitch) so that the 16-byte fragment reads of a quarter-wave fall on
//           distinct LDS banks;
//   W tile  4 n-tiles x 4 k-tiles already in fragment order, copied verbatim
//           (a fragment read is 1 KiB contiguous).
// Each wave accumulates a 64 x 64 block as 2 x 2 MFMA 32x32x16 tiles in fp32.
#pragma once

#include "common.h"

namespace ernie {

constexpr int kGemmBM = 128, kGemmBN = 128, kGemmBK = 64;
constexpr int kGemmAPitch = kGemmBK + 8;                       // halves
constexpr int kGemmAStage = kGemmBM * kGemmAPitch;             // halves
constexpr int kGemmBStage = (kGemmBN / 32) * (kGemmBK / 16) * 512;   // halves
constexpr int kGemmLdsBytes = 2 * (kGemmAStage + kGemmBStage) * 2;

// ---- epilogues: called once per accumulator element with (row, col, value incl. bias)

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

template <class Epi>
__global__ __launch_bounds__(256) void gemm_prefill_kernel(const half_t* __restrict__ A,
                                                           const half_t* __restrict__ Wp,
                                                           const float* __restrict__ bias, int M, int N, int K,
                                                           int n_tiles32, int tiles_n, Epi epi) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);
  half_t* sB = sA + 2 * kGemmAStage;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int wm = wave >> 1, wn = wave & 1;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int m0 = tile_m * kGemmBM, n0 = tile_n * kGemmBN;
  const int k_tiles = K / 16;
  const int steps = K / kGemmBK;

  // global -> register staging: 4 A chunks and 4 W chunks of 16 bytes per thread
  half8 ra[4], rb[4];
  auto load_global = [&](int step) {
    const int k0 = step * kGemmBK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i;
      const int r = id >> 3, cc = id & 7;
      const int gm = m0 + r;
      half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (gm < M) v = *reinterpret_cast<const half8*>(A + (size_t)gm * K + k0 + cc * 8);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int nt = n0 / 32 + i;          // thread tid copies chunk tid of n-tile i (4 KiB per n-tile)
      half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (nt < n_tiles32)
        v = *reinterpret_cast<const half8*>(Wp + packed_frag_offset(nt, k0 / 16, k_tiles) + tid * 8);
      rb[i] = v;
    }
  };
  auto store_lds = [&](int buf) {
    half_t* a = sA + buf * kGemmAStage;
    half_t* b = sB + buf * kGemmBStage;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i;
      const int r = id >> 3, cc = id & 7;
      *reinterpret_cast<half8*>(a + r * kGemmAPitch + cc * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<half8*>(b + i * 2048 + tid * 8) = rb[i];
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int step = 0; step < steps; ++step) {
    const int buf = step & 1;
    if (step + 1 < steps) load_global(step + 1);
    const half_t* a = sA + buf * kGemmAStage + (wm * 64 + (lane & 31)) * kGemmAPitch + 8 * (lane >> 5);
    const half_t* b = sB + buf * kGemmBStage + (wn * 2) * 2048 + lane * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      half8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const half8*>(a + i * 32 * kGemmAPitch + ks * 16);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const half8*>(b + j * 2048 + ks * 512);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
    }
    if (step + 1 < steps) store_lds(buf ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = n0 + wn * 64 + j * 32 + (lane & 31);
    if (col >= N) continue;
    const float bv = bias[col];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + i * 32 + mfma32_row(v, lane);
        if (row < M) epi(row, col, acc[i][j][v] + bv);
      }
  }
}

}  // namespace ernie

// Decode-step GEMM: out[B, N] = x[B, K] * W[N, K]^T for a small number of rows
// (B <= 256).  The work is streaming W once from HBM, so the kernel is built
// around fully coalesced weight reads:
//   - W is fragment-major: one 32-column x 16-k fragment is 1 KiB contiguous
//     and is fetched by one wave with a single 16-byte load per lane;
//   - one workgroup owns one 32-column strip; its NW waves split K, each wave
//     keeps MT = ceil(B / 32) accumulator tiles (MFMA 32x32x16, fp32) and reuses
//     every weight fragment for all MT row tiles;
//   - the waves' partial tiles are summed through LDS in a fixed order
//     (deterministic), then the epilogue runs on the finished strip.
#pragma once

#include "common.h"

namespace ernie {

// ---- epilogues: operate on one finished 32-row x 32-col tile held in the MFMA
// D layout by one wave (row = 32 * mt + mfma32_row(v, lane), col = n0 + lane % 32).

// QKV: + bias; Q -> q[B][d] (fp16); K, V appended to the cache at slot cache_len[b].
struct SkinnyQKV {
  half_t* q;             // [B, d]
  half_t* kcache;        // layer base [Bmax][H][S][64]
  half_t* vcache;
  const int* cache_len;  // [B]
  int d, H, S;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    const int part = col / d, within = col - part * d;
    if (part == 0) {
      q[(size_t)row * d + within] = (half_t)v;
    } else {
      const int pos = cache_len[row];
      if (pos < S) {
        half_t* base = (part == 1) ? kcache : vcache;
        base[(((size_t)row * H + (within >> 6)) * S + pos) * 64 + (within & 63)] = (half_t)v;
      }
    }
  }
};

// out-projection / FFN2: Y = acc + bias + residual, kept in fp32 for the LayerNorm that follows.
struct SkinnyResidual {
  const half_t* res;   // [B, N] fp16
  float* y;            // [B, N] fp32
  int N;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    const size_t o = (size_t)row * N + col;
    y[o] = v + (float)res[o];
  }
};

struct SkinnyGelu {
  half_t* g;
  int N;
  __device__ __forceinline__ void operator()(int row, int col, float v) const {
    g[(size_t)row * N + col] = (half_t)gelu_erf(v);
  }
};

template <int MT, int NW, class Epi>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(const half_t* __restrict__ X,
                                                              const half_t* __restrict__ Wp,
                                                              const float* __restrict__ bias, int B, int N, int K,
                                                              Epi epi) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float* red = reinterpret_cast<float*>(smem_raw);   // [NW][MT][16][64]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
  const int nt = blockIdx.x;
  const int k_tiles = K / 16;
  // balanced contiguous split of the k-tiles over the waves
  const int kb = (int)(((long long)k_tiles * wave) / NW);
  const int ke = (int)(((long long)k_tiles * (wave + 1)) / NW);

  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;

  const half_t* wp = Wp + packed_frag_offset(nt, 0, k_tiles) + lane * 8;
  const int xr = lane & 31, xk = 8 * (lane >> 5);

  int kt = kb;
  for (; kt + 4 <= ke; kt += 4) {
    half8 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = *reinterpret_cast<const half8*>(wp + (size_t)(kt + u) * 512);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int row = m * 32 + xr;
      half8 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        x[u] = (row < B) ? *reinterpret_cast<const half8*>(X + (size_t)row * K + (kt + u) * 16 + xk) : z;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[m] = mfma32(x[u], w[u], acc[m]);
    }
  }
  for (; kt < ke; ++kt) {
    const half8 w = *reinterpret_cast<const half8*>(wp + (size_t)kt * 512);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int row = m * 32 + xr;
      half8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row < B) x = *reinterpret_cast<const half8*>(X + (size_t)row * K + kt * 16 + xk);
      acc[m] = mfma32(x, w, acc[m]);
    }
  }

  // cross-wave reduction in a fixed order: wave w finishes row tiles m with m % NW == w
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  __syncthreads();

  const int col = nt * 32 + (lane & 31);
  const float bv = (col < N) ? bias[col] : 0.f;
  for (int m = wave; m < MT; m += NW) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[((w * MT + m) * 16 + v) * 64 + lane];
      const int row = m * 32 + mfma32_row(v, lane);
      if (row < B && col < N) epi(row, col, s + bv);
    }
  }
}

// Output projection onto the trimmed word-embedding table with the first
// argmax stage fused: each strip of 32 vocabulary rows reports, per sequence,
// its best (logit, index); logits are optionally written out in fp32.
// Columns >= N (padding of the last strip) never win.
template <int MT, int NW>
__global__ __launch_bounds__(NW * 64) void logits_argmax_kernel(const half_t* __restrict__ X,
                                                                const half_t* __restrict__ Ep, int B, int N,
                                                                int K, float* __restrict__ logits_out,
                                                                float* __restrict__ strip_val,
                                                                int* __restrict__ strip_idx, int strips) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float* red = reinterpret_cast<float*>(smem_raw);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
  const int nt = blockIdx.x;
  const int k_tiles = K / 16;
  const int kb = (int)(((long long)k_tiles * wave) / NW);
  const int ke = (int)(((long long)k_tiles * (wave + 1)) / NW);

  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;

  const half_t* wp = Ep + packed_frag_offset(nt, 0, k_tiles) + lane * 8;
  const int xr = lane & 31, xk = 8 * (lane >> 5);
  for (int kt = kb; kt < ke; ++kt) {
    const half8 w = *reinterpret_cast<const half8*>(wp + (size_t)kt * 512);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const int row = m * 32 + xr;
      half8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row < B) x = *reinterpret_cast<const half8*>(X + (size_t)row * K + kt * 16 + xk);
      acc[m] = mfma32(x, w, acc[m]);
    }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  __syncthreads();

  const int col = nt * 32 + (lane & 31);
  for (int m = wave; m < MT; m += NW) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) s += red[((w * MT + m) * 16 + v) * 64 + lane];
      const int row = m * 32 + mfma32_row(v, lane);
      if (logits_out && row < B && col < N) logits_out[(size_t)row * N + col] = s;
      // best of this strip for `row`: reduce over the 32 lanes that share lane / 32
      float bv = (col < N) ? s : -INFINITY;
      int bi = col;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        argmax_merge(bv, bi, ov, oi);
      }
      if ((lane & 31) == 0 && row < B) {
        strip_val[(size_t)row * strips + nt] = bv;
        strip_idx[(size_t)row * strips + nt] = bi;
      }
    }
  }
}

}  // namespace ernie

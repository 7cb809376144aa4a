// Latency-oriented decode-step kernels for small batches (B <= 64).
//
// At B = 32 one decode step moves only 1-5 MB per GEMM, so a step is bound by
// the number of dependent phases, not by any single kernel.  These kernels cut
// a layer to five phases by moving every row-wise operation into the PROLOGUE
// of its consumer:
//
//   gemm_dec<PRO_LN>    A = LayerNorm(sum_k partial_k + bias + residual)     (QKV, FFN1)
//   gemm_dec<PRO_GELU>  A = gelu(raw + bias)                                 (FFN2)
//   gemm_dec<PRO_PLAIN> A = fp16 activations                                 (out-proj, logits)
//   attn_decode_fused   q, k, v = raw + bias; append k, v; attend            (attention)
//
// Every GEMM phase writes raw fp32 accumulators (optionally split over K into
// `gridDim.y` partial buffers that the consumer adds in a fixed order), so the
// result does not depend on scheduling.  Each workgroup issues its weight
// fragment loads BEFORE the prologue: the HBM latency of the weight stream
// hides under the L2-resident activation work.
#pragma once

#include "common.h"
#include "rowops.h"

namespace ernie {

enum { PRO_PLAIN = 0, PRO_LN = 1, PRO_GELU = 2 };
enum { EPI_RAW = 0, EPI_ARGMAX = 1 };

constexpr int kDecMaxFrag = 8;   // weight fragments a wave keeps in flight

struct DecGemmArgs {
  const half_t* Wp;   // packed [N, K]
  int N, K, B;
  // prologue inputs
  const half_t* a16;  // PRO_PLAIN: [B, K] fp16
  const float* r32;   // PRO_LN / PRO_GELU: raw fp32 [sk_in][B][K]
  int sk_in;
  const float* bias;  // [K] bias of the GEMM that produced r32
  const half_t* res;  // PRO_LN: residual [B, K] fp16
  const float* gamma;
  const float* beta;
  float eps;
  half_t* xout;       // PRO_LN: normalised rows [B, K] fp16, written by workgroup (0, 0); may be null
  // outputs
  float* rout;        // EPI_RAW: [gridDim.y][B][N]
  float* logits_out;  // EPI_ARGMAX: [B, N] or null
  float* strip_val;   // EPI_ARGMAX: [B, strips]
  int* strip_idx;
  int strips;
};

template <int MT, int NW, int PRO, int EPI, int RC>
__global__ __launch_bounds__(NW * 64) void gemm_dec_kernel(DecGemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  half_t* sA = reinterpret_cast<half_t*>(smem_raw);
  float* red = reinterpret_cast<float*>(smem_raw);   // reused after the MFMA loop

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nt = blockIdx.x;
  const int K = p.K, B = p.B;
  const int k_tiles = K / 16;
  const int tiles_wg = k_tiles / gridDim.y;           // host guarantees divisibility
  const int tile0 = blockIdx.y * tiles_wg;
  const int kslice = tiles_wg * 16, k0 = tile0 * 16;
  const int pitch = kslice + 8;
  const int kb = tiles_wg * wave / NW, ke = tiles_wg * (wave + 1) / NW;

  // 1. weight stream: first batch of fragments in flight before anything else
  const half_t* wp = p.Wp + packed_frag_offset(nt, tile0, k_tiles) + lane * 8;
  half8 wf[kDecMaxFrag];
#pragma unroll
  for (int u = 0; u < kDecMaxFrag; ++u) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    wf[u] = (kb + u < ke) ? *reinterpret_cast<const half8*>(wp + (size_t)(kb + u) * 512) : z;
  }

  // 2. prologue: build the fp16 A tile [MT * 32, kslice] in LDS
  if constexpr (PRO == PRO_LN) {
    const int chunks = K / 8;
    for (int r = wave; r < MT * 32; r += NW) {
      RowRegs<RC> v;
      if (r < B) {
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const int ch = c * 64 + lane;
          if (ch < chunks) {
            const half8 rs = *reinterpret_cast<const half8*>(p.res + (size_t)r * K + ch * 8);
            const float4 b0 = *reinterpret_cast<const float4*>(p.bias + ch * 8);
            const float4 b1 = *reinterpret_cast<const float4*>(p.bias + ch * 8 + 4);
            float a[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
            for (int s = 0; s < p.sk_in; ++s) {
              const float* src = p.r32 + ((size_t)s * B + r) * K + ch * 8;
              const float4 x0 = *reinterpret_cast<const float4*>(src);
              const float4 x1 = *reinterpret_cast<const float4*>(src + 4);
              a[0] += x0.x; a[1] += x0.y; a[2] += x0.z; a[3] += x0.w;
              a[4] += x1.x; a[5] += x1.y; a[6] += x1.z; a[7] += x1.w;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) v.v[c][j] = a[j] + (float)rs[j];
          }
        }
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < RC; ++c)
          if (c * 64 + lane < chunks)
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v.v[c][j];
        const float mean = wave_sum(s) / (float)K;
        float q = 0.f;
#pragma unroll
        for (int c = 0; c < RC; ++c)
          if (c * 64 + lane < chunks)
#pragma unroll
            for (int j = 0; j < 8; ++j) { const float t = v.v[c][j] - mean; q += t * t; }
        const float rstd = rsqrtf(wave_sum(q) / (float)K + p.eps);
        const bool writer = p.xout && blockIdx.x == 0 && blockIdx.y == 0;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
          const int ch = c * 64 + lane;
          if (ch < chunks) {
            half8 o;
#pragma unroll
            for (int j = 0; j < 8; ++j)
              o[j] = (half_t)((v.v[c][j] - mean) * rstd * p.gamma[ch * 8 + j] + p.beta[ch * 8 + j]);
            const int kk = ch * 8 - k0;
            if (kk >= 0 && kk < kslice) *reinterpret_cast<half8*>(sA + r * pitch + kk) = o;
            if (writer) *reinterpret_cast<half8*>(p.xout + (size_t)r * K + ch * 8) = o;
          }
        }
      } else {
        for (int kk = lane * 8; kk < kslice; kk += 512) {
          const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
          *reinterpret_cast<half8*>(sA + r * pitch + kk) = z;
        }
      }
    }
  } else {
    const int chunks = kslice / 8;
    for (int id = tid; id < MT * 32 * chunks; id += NW * 64) {
      const int r = id / chunks, ch = id - r * chunks;
      half8 o = {0, 0, 0, 0, 0, 0, 0, 0};
      if (r < B) {
        if constexpr (PRO == PRO_PLAIN) {
          o = *reinterpret_cast<const half8*>(p.a16 + (size_t)r * K + k0 + ch * 8);
        } else {
          const float* src = p.r32 + (size_t)r * K + k0 + ch * 8;
          const float* bs = p.bias + k0 + ch * 8;
          const float4 x0 = *reinterpret_cast<const float4*>(src), x1 = *reinterpret_cast<const float4*>(src + 4);
          const float4 b0 = *reinterpret_cast<const float4*>(bs), b1 = *reinterpret_cast<const float4*>(bs + 4);
          o[0] = (half_t)gelu_erf(x0.x + b0.x); o[1] = (half_t)gelu_erf(x0.y + b0.y);
          o[2] = (half_t)gelu_erf(x0.z + b0.z); o[3] = (half_t)gelu_erf(x0.w + b0.w);
          o[4] = (half_t)gelu_erf(x1.x + b1.x); o[5] = (half_t)gelu_erf(x1.y + b1.y);
          o[6] = (half_t)gelu_erf(x1.z + b1.z); o[7] = (half_t)gelu_erf(x1.w + b1.w);
        }
      }
      *reinterpret_cast<half8*>(sA + r * pitch + ch * 8) = o;
    }
  }
  __syncthreads();

  // 3. MFMA over this wave's k-tiles
  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;
  const half_t* ap = sA + (lane & 31) * pitch + 8 * (lane >> 5);
  for (int base = kb; base < ke; base += kDecMaxFrag) {
#pragma unroll
    for (int u = 0; u < kDecMaxFrag; ++u) {
      if (base + u < ke) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const half8 a = *reinterpret_cast<const half8*>(ap + m * 32 * pitch + (base + u) * 16);
          acc[m] = mfma32(a, wf[u], acc[m]);
        }
      }
    }
    if (base + kDecMaxFrag < ke) {
#pragma unroll
      for (int u = 0; u < kDecMaxFrag; ++u) {
        const int kt = base + kDecMaxFrag + u;
        const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        wf[u] = (kt < ke) ? *reinterpret_cast<const half8*>(wp + (size_t)kt * 512) : z;
      }
    }
  }
  __syncthreads();          // all waves are done reading sA before it is reused

  // 4. cross-wave reduction in a fixed order
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  __syncthreads();

  const int col = nt * 32 + (lane & 31);
  // (m, v) pairs are dealt to the waves so that every wave takes part in the epilogue
  for (int mv = wave; mv < MT * 16; mv += NW) {
    const int m = mv >> 4, v = mv & 15;
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[((w * MT + m) * 16 + v) * 64 + lane];
    const int row = m * 32 + mfma32_row(v, lane);
    if constexpr (EPI == EPI_RAW) {
      if (row < B && col < p.N) p.rout[((size_t)blockIdx.y * B + row) * p.N + col] = s;
    } else {
      if (p.logits_out && row < B && col < p.N) p.logits_out[(size_t)row * p.N + col] = s;
      float bv = (col < p.N) ? s : -INFINITY;
      int bi = col;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        argmax_merge(bv, bi, ov, oi);
      }
      if ((lane & 31) == 0 && row < B) {
        p.strip_val[(size_t)row * p.strips + nt] = bv;
        p.strip_idx[(size_t)row * p.strips + nt] = bi;
      }
    }
  }
}

// X = LayerNorm(sum_k partial_k + bias + residual), one wave per row (used once per step, before the logits).
template <int RC>
__global__ __launch_bounds__(256) void ln_partials_kernel(const float* __restrict__ r32, int sk_in,
                                                          const float* __restrict__ bias,
                                                          const half_t* __restrict__ res, int rows, int d,
                                                          const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float eps,
                                                          half_t* __restrict__ X, float* __restrict__ hidden_out) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  RowRegs<RC> v;
  const int chunks = d / 8;
#pragma unroll
  for (int c = 0; c < RC; ++c) {
    const int ch = c * 64 + lane;
    if (ch < chunks) {
      const half8 rs = *reinterpret_cast<const half8*>(res + (size_t)r * d + ch * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) v.v[c][j] = bias[ch * 8 + j] + (float)rs[j];
      for (int s = 0; s < sk_in; ++s) {
        const float* src = r32 + ((size_t)s * rows + r) * d + ch * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) v.v[c][j] += src[j];
      }
    }
  }
  row_layernorm_store(v, d, lane, gamma, beta, eps, X + (size_t)r * d);
  if (hidden_out) {
    // the caller's fp32 copy is the fp16 value that feeds the projection, widened
#pragma unroll
    for (int c = 0; c < RC; ++c) {
      const int ch = c * 64 + lane;
      if (ch < chunks) {
        const half8 o = *reinterpret_cast<const half8*>(X + (size_t)r * d + ch * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) hidden_out[(size_t)r * d + ch * 8 + j] = (float)o[j];
      }
    }
  }
}

}  // namespace ernie

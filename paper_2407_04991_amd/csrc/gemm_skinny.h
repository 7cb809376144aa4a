// Output projection for large batches (B > 64): logits[B, V'] = x[B, d] * E'^T with the first argmax
// stage fused.  The table is fragment-major (one 32-row x 16-k fragment = 1 KiB contiguous, fetched with
// one 16-byte load per lane); a workgroup owns a strip of 32 vocabulary rows, its NW waves split K, every
// wave keeps MT = ceil(B / 32) accumulator tiles and reuses each table fragment for all of them; the
// waves' tiles are summed through LDS in a fixed order.  Activations are read straight from global
// memory (they do not fit in LDS at this batch size).
#pragma once

#include "common.h"

namespace ernie {

// Output projection onto the trimmed word-embedding table with the first
// argmax stage fused: each strip of 32 vocabulary rows reports, per sequence,
// its best (logit, index); logits are optionally written out in fp32.
// Columns >= N (padding of the last strip) never win.
template <int MT, int NW>
__global__ __launch_bounds__(NW * 64) void logits_argmax_kernel(const half_t* __restrict__ X,
                                                                const half_t* __restrict__ Ep, int B, int N,
                                                                int K, const float* __restrict__ out_bias,
                                                                float* __restrict__ logits_out,
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
      if (out_bias && col < N) s += out_bias[col];            // optional output bias of the projection
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

// First argmax stage over whole rows, for projections computed by the MFMA GEMM pipeline as fp32 partial
// logits [sk][B][N]: one workgroup per sequence adds the partials in index order (+ optional output bias),
// optionally writes the logits out, and reports the row's best (value, index) as a single "strip"
// candidate for argmax_final_kernel (strips = 1).  N must be a multiple of 4 and the buffers 16-byte aligned.
__global__ __launch_bounds__(256) void logits_rows_argmax_kernel(const float* __restrict__ part, int sk, int B, int N,
                                                                 const float* __restrict__ out_bias,
                                                                 float* __restrict__ logits_out,
                                                                 float* __restrict__ cand_val, int* __restrict__ cand_idx) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* row = part + (size_t)b * N;
  const size_t slab = (size_t)B * N;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  // N is a multiple of 8 on this path (the GEMM epilogue stores runs of 8 columns): 16-byte pieces, four per
  // thread requested together (addresses clamped, not predicated; a loop of load + compare per piece costs a
  // memory round trip per trip).  The host splits this projection at most two ways; further partials are added
  // by the general loop.
  for (int c0 = tid * 4; c0 < N; c0 += 4096) {
    float4 z[4], y[4], ob[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = min(c0 + q * 1024, N - 4);
      z[q] = *reinterpret_cast<const float4*>(row + c);
      y[q] = *reinterpret_cast<const float4*>(row + (size_t)(sk > 1 ? 1 : 0) * slab + c);
      ob[q] = out_bias ? *reinterpret_cast<const float4*>(out_bias + c) : float4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + q * 1024;
      if (c >= N) break;
      float4 a = z[q];
      if (sk > 1) { a.x += y[q].x; a.y += y[q].y; a.z += y[q].z; a.w += y[q].w; }
      for (int s = 2; s < sk; ++s) {
        const float4 t = *reinterpret_cast<const float4*>(row + (size_t)s * slab + c);
        a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
      }
      a.x += ob[q].x; a.y += ob[q].y; a.z += ob[q].z; a.w += ob[q].w;
      if (logits_out) *reinterpret_cast<float4*>(logits_out + (size_t)b * N + c) = a;
      argmax_merge(bv, bi, a.x, c); argmax_merge(bv, bi, a.y, c + 1);
      argmax_merge(bv, bi, a.z, c + 2); argmax_merge(bv, bi, a.w, c + 3);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    argmax_merge(bv, bi, ov, oi);
  }
  if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w) argmax_merge(bv, bi, sv[w], si[w]);
    cand_val[b] = bv;
    cand_idx[b] = bi;
  }
}

}  // namespace ernie

// Measurement kernel behind ernie_debug_handover: G persistent workgroups run S dependent all-to-all stages.  In
// every stage a workgroup publishes `out16` 16-byte units and then reads `PIECES` units per thread spread over what
// ALL workgroups published in the stage before.  Two hand-over protocols:
//   mode 0  tagged pairs, as the one-launch decode kernel uses them: {payload, tag, payload, tag} written with
//           agent-scope stores, read with agent-scope loads until both tags of a unit match (no fence, no flag)
//   mode 1  fence and flag: plain stores, __threadfence() (an L2 write-back on this part), one flag per workgroup;
//           the consumer polls all flags, fences again (an L2 invalidate) and reads with plain loads
// Every payload is checked against its closed form, so a protocol that let stale data through would be counted.
#pragma once

#include "decode_persist.h"

namespace ernie {

constexpr int kProbeThreads = 512;

template <int MODE, int PIECES>
__global__ __launch_bounds__(kProbeThreads) void handover_probe_kernel(unsigned* bufs, unsigned buf_units, unsigned* flags,
                                                                      int S, int out16, unsigned epoch0, unsigned spin_limit,
                                                                      int* gave_up, unsigned* bad) {
  const int tid = threadIdx.x, wg = blockIdx.x, G = gridDim.x;
  const unsigned total16 = (unsigned)G * out16;
  __shared__ int s_fail;
  if (tid == 0) s_fail = 0;
  lds_barrier();
  unsigned nbad = 0;
  for (int s = 0; s < S; ++s) {
    const unsigned epoch = epoch0 + s;
    unsigned* out = bufs + (size_t)(s % 3) * buf_units * 4;
    const unsigned* in = bufs + (size_t)((s + 2) % 3) * buf_units * 4;
    const __amdgpu_buffer_rsrc_t rin = xch_rsrc(in, buf_units * 16), rout = xch_rsrc(out, buf_units * 16);
    if (s > 0) {
      bool fail = false;
      if (MODE == 1) {
        if (tid < 64 && tid * 4 < G) {
          const __amdgpu_buffer_rsrc_t rf = xch_rsrc(flags, 1024 * 4);
          unsigned spins = 0;
          while (true) {
            asm volatile("" ::: "memory");
            const u32x4 f = xch_load16(rf, tid * 16);
            bool all = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) if (tid * 4 + j < G && (int)(f[j] - (epoch - 1)) < 0) all = false;
            if (all) break;
            if (++spins > spin_limit) { fail = true; break; }
          }
        }
        if (persist_sync_fail(fail, &s_fail)) break;
        __threadfence();
      }
      u32x4 v[PIECES];
      unsigned idx[PIECES];
#pragma unroll
      for (int q = 0; q < PIECES; ++q)      // 1 KiB contiguous per wave and piece, the pieces spread over all producers
        idx[q] = (unsigned)((((size_t)(wg * 131 + q * 8 + (tid >> 6)) * 2654435761u) % (total16 / 64)) * 64 + (tid & 63));
      if (MODE == 0) {
        unsigned spins = 0;
        while (true) {
          asm volatile("" ::: "memory");
          bool ok = true;
#pragma unroll
          for (int q = 0; q < PIECES; ++q) v[q] = xch_load16(rin, idx[q] * 16);
#pragma unroll
          for (int q = 0; q < PIECES; ++q) ok &= v[q][1] == epoch - 1 && v[q][3] == epoch - 1;
          if (__all(ok)) break;
          if (++spins > spin_limit) { fail = true; break; }
        }
      } else {
#pragma unroll
        for (int q = 0; q < PIECES; ++q) v[q] = *reinterpret_cast<const u32x4*>(in + (size_t)idx[q] * 4);
      }
      if (persist_sync_fail(fail, &s_fail)) break;
#pragma unroll
      for (int q = 0; q < PIECES; ++q) {
        const unsigned want = idx[q] ^ ((epoch - 1) * 0x9e3779b9u);
        if (v[q][0] != want || v[q][2] != ~want) ++nbad;
      }
    }
    for (int i = tid; i < out16; i += kProbeThreads) {
      const unsigned idx = (unsigned)wg * out16 + i;
      const unsigned p0 = idx ^ (epoch * 0x9e3779b9u);
      if (MODE == 0) xch_store16(rout, idx * 16, p0, ~p0, epoch);
      else { const u32x4 o = {p0, epoch, ~p0, epoch}; *reinterpret_cast<u32x4*>(out + (size_t)idx * 4) = o; }
    }
    if (MODE == 1) {
      __threadfence();
      __syncthreads();
      if (tid == 0) __hip_atomic_store(flags + wg, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (s_fail && tid == 0) *gave_up = 1;
  if (nbad) atomicAdd(bad, nbad);
}

}  // namespace ernie

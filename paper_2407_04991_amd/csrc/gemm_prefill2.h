// Prefill GEMM on FP16 MFMA, asynchronous-copy pipeline:
//   C[M, N] = A[M, K] * W[N, K]^T  (+ fused epilogue), fp32 accumulation.
//
// One workgroup (WGM x WGN waves, each 32 TM x 32 TN outputs as 2 TM x 2 TN tiles of the 16x16x32 MFMA) owns a
// (32 WGM TM) x (32 WGN TN) output tile and walks K in steps of BK through an
// S-stage ring in LDS.  The 16x16x32 instruction is used because it moves a third fewer register bytes per
// flop than 32x32x16 (accumulators are read and written once per 32 instead of per 16 of K): in a
// register-only loop on random operands, where the chip is power-limited, it sustains 1.95 PFLOP/s against
// 1.45.  Operands travel global -> LDS
// directly (global_load_lds_dwordx4: lane l's 16 bytes land at LDS base + 16 l),
// so no registers are spent on staging and S - 1 stages stay in flight per wave.
//
//   A stage  32 WGM TM rows x BK halves.  BK = 64: row-major rows of 128 bytes, 16-byte chunk c of row r in
//            slot c ^ ((r / 2) % 8).  BK = 32: the 16 rows x 4 chunks that one load instruction covers are
//            permuted inside their 1 KiB block so that every chunk sits on the banks it would have in rows of
//            128 bytes (position ((r / 2) % 4) * 16 + (r % 2) * 8 + (c ^ ((r / 2) % 8)), in 16-byte units).
//            Both are conflict-free for the 16 x 32 operand read (lane -> row lane % 16, chunk lane / 16),
//            measured at 230 B/clk/CU; plain rows of 64 bytes with a 4-way XOR ran that read at half rate.
//            The lanes that fetch one row are adjacent, so a row is still one contiguous 64/128-byte run.
//   W stage  the packed weight (1 KiB fragments of 32 columns x 16 k, see common.h) is copied verbatim; a
//            16-column x 32-k operand is one half (columns) of two consecutive fragments (k), still one
//            16-byte read per lane, every quarter-wave on 256 contiguous bytes.
//
// Rows >= M and n-tiles past the end are clamped to the last valid one (their
// products land in accumulator entries the epilogue never stores).
#pragma once

#include <type_traits>

#include "common.h"
#include "gemm_prefill.h"   // epilogue functors

namespace ernie {

typedef __attribute__((address_space(1))) const void global_cptr_t;
typedef __attribute__((address_space(3))) void lds_ptr_t;

__device__ __forceinline__ void async_copy16(const void* gsrc, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((global_cptr_t*)gsrc, (lds_ptr_t*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits [3:0] and [15:14]).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// An epilogue that reads memory (a residual) declares load8(row, col) -> half8 and takes the loaded value as
// a fourth argument of store8: the kernel then issues every such load of a wave before the first store, so
// that they are in flight together instead of one dependent round trip per 8 outputs.
template <class E, class = void>
struct epi_has_load { static constexpr bool value = false; };
template <class E>
struct epi_has_load<E, decltype((void)&E::load8)> { static constexpr bool value = true; };

template <int WGM, int WGN, int TM, int TN, int BK, int S>
struct GemmPipe {
  static constexpr int kWaves = WGM * WGN;                   // WGM x WGN waves, each TM x TN MFMA tiles
  static constexpr int kBM = 32 * WGM * TM, kBN = 32 * WGN * TN;
  static constexpr int kRowBytes = BK * 2;
  static constexpr int kChunks = kRowBytes / 16;             // 16-byte chunks per A row (4 or 8)
  static constexpr int kRowsPer256 = 256 / kRowBytes;        // rows sharing one 64-bank line (4 or 2)
  static constexpr int kRowsPerInstr = 64 / kChunks;         // rows one load instruction covers (16 or 8)
  static constexpr int kAInstr = kBM / kRowsPerInstr / kWaves;   // A load instructions per wave per stage
  static constexpr int kBFrags = (kBN / 32) * (BK / 16);     // W fragments per stage
  static constexpr int kBInstr = (kBFrags + kWaves - 1) / kWaves;   // W load instructions per wave per stage
  static constexpr int kLoads = kAInstr + kBInstr;           // outstanding loads per wave per stage
  static constexpr int kAStage = kBM * kRowBytes;            // bytes
  static constexpr int kBStage = kBInstr * kWaves * 1024;    // bytes (rounded up to whole instructions)
  static constexpr int kStage = kAStage + kBStage;
  static constexpr int kLdsBytes = S * kStage;
  static_assert(kAInstr >= 1 && kBM % (kRowsPerInstr * kWaves) == 0, "A tile must split evenly over the waves");
};

// DBG (measurement builds only, 0 in the library): 8 = no A copies, 16 = no W copies.
template <int WGM, int WGN, int TM, int TN, int BK, int S, class Epi, int DBG = 0>
__global__ __launch_bounds__(64 * WGM * WGN, (TM * TN <= 8 ? 2 : 1)) void gemm_prefill2_kernel(const half_t* __restrict__ A,
                                                            const half_t* __restrict__ Wp,
                                                            const float* __restrict__ bias, int M, int N, int K,
                                                            int n_tiles32, int tiles_n, Epi epi) {
  using P = GemmPipe<WGM, WGN, TM, TN, BK, S>;
  extern __shared__ __align__(16) unsigned char smem_raw[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int tile = xcd_contiguous_id(blockIdx.x, gridDim.x);
  // tiles_n > 0: column tiles fastest (neighbouring workgroups of an XCD share A rows: prefill, M large);
  // tiles_n < 0: -tiles_n row tiles, fastest (the few row tiles of a weight column strip run next to each other
  // in one XCD and fetch the strip once: decode at large batch)
  int tile_m, tile_n;
  if (tiles_n > 0) { tile_m = tile / tiles_n; tile_n = tile - tile_m * tiles_n; }
  else { tile_n = tile / (-tiles_n); tile_m = tile + tile_n * tiles_n; }
  const int m0 = tile_m * P::kBM, n0 = tile_n * P::kBN;
  const int k_tiles = K / 16;
  // gridDim.y > 1 splits the contraction: workgroup y accumulates k in [y, y + 1) * K / gridDim.y and the
  // epilogue functor routes the partial result by blockIdx.y (host guarantees divisibility by BK)
  const int steps = K / BK / gridDim.y;
  const int kbeg = blockIdx.y * steps * BK;

  // bias of this lane's TN columns: fetched now, so that the epilogue does not start with a memory round trip
  float bvv[2 * TN];
#pragma unroll
  for (int j = 0; j < 2 * TN; ++j) {
    const int mycol = n0 + wn * 32 * TN + j * 16 + (lane & 15);
    bvv[j] = (mycol < N) ? bias[mycol] : 0.f;
  }

  // ---- per-lane source addresses of this wave's load instructions (k offset added per step)
  const half_t* a_src[P::kAInstr];
#pragma unroll
  for (int i = 0; i < P::kAInstr; ++i) {
    int r, c;      // row inside the tile and 16-byte chunk of it that this lane's copy lands on (LDS position = lane)
    if constexpr (BK == 32) {
      // 16 rows x 4 chunks per instruction: chunk c of row r sits at 16-byte position
      //   ((r / 2) % 4) * 16 + (r % 2) * 8 + (c ^ ((r / 2) % 8))
      // of its 1 KiB block, i.e. on the banks it would have in rows of 128 bytes (see the W / A stage notes above)
      const int line = lane >> 4, u = lane & 15, x = u & 7;
      r = (wave * P::kAInstr + i) * 16 + 2 * (line + 4 * (x >> 2)) + (u >> 3);
      c = (x & 3) ^ line;
    } else {
      r = (wave * P::kAInstr + i) * P::kRowsPerInstr + lane / P::kChunks;
      c = (lane % P::kChunks) ^ ((r / P::kRowsPer256) % P::kChunks);                  // global chunk that lands in slot lane % kChunks
    }
    a_src[i] = A + (size_t)min(m0 + r, M - 1) * K + kbeg + c * 8;
  }
  // W fragment f of a stage = (n-tile f / (BK/16), k-tile f % (BK/16)); wave w copies fragments w*kBInstr + j
  const half_t* b_src[P::kBInstr];
#pragma unroll
  for (int j = 0; j < P::kBInstr; ++j) {
    const int f = min(wave * P::kBInstr + j, P::kBFrags - 1);
    const int nt = min(n0 / 32 + f / (BK / 16), n_tiles32 - 1);
    b_src[j] = Wp + packed_frag_offset(nt, kbeg / 16 + f % (BK / 16), k_tiles) + lane * 8;
  }

  auto issue = [&](int stage, int kstep) {
    unsigned char* sa = smem_raw + stage * P::kStage;
    unsigned char* sb = sa + P::kAStage;
    const int k0 = kstep * BK;
    if constexpr (!(DBG & 8)) {
#pragma unroll
      for (int i = 0; i < P::kAInstr; ++i)
        async_copy16(a_src[i] + k0, sa + (wave * P::kAInstr + i) * P::kRowsPerInstr * P::kRowBytes);
    }
    if constexpr (!(DBG & 16)) {
#pragma unroll
      for (int j = 0; j < P::kBInstr; ++j)
        async_copy16(b_src[j] + (size_t)(k0 / 16) * 512, sb + (wave * P::kBInstr + j) * 1024);
    }
  };

  floatx4 acc[2 * TM][2 * TN];
#pragma unroll
  for (int i = 0; i < 2 * TM; ++i)
#pragma unroll
    for (int j = 0; j < 2 * TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // ---- fragment read offsets (bytes) inside a stage.  A operand of sub-tile i: lane l holds row 16 i + l % 16,
  // k = 8 (l / 16) .. + 7 of a 32-wide k step; W operand of sub-tile j: column 16 j + l % 16, same k.
  const int l16 = lane & 15, kq = lane >> 4;
  int a_off[2 * TM], a_swz[2 * TM];
#pragma unroll
  for (int i = 0; i < 2 * TM; ++i) {
    const int r = wm * 32 * TM + i * 16 + l16;
    if constexpr (BK == 32) {
      const int rl = r & 15;                                   // r is a multiple of 16 plus l16
      a_off[i] = (r >> 4) * 1024 + (((rl >> 1) & 3) * 16 + (rl & 1) * 8) * 16;
      a_swz[i] = (rl >> 1) & 7;
    } else {
      a_off[i] = r * P::kRowBytes;
      a_swz[i] = (r / P::kRowsPer256) % P::kChunks;
    }
  }
  // 16-k fragment t of a 32-k step holds k-quarters 2 t and 2 t + 1 in its two 512-byte halves
  const int b_lane = (kq >> 1) * 1024 + (kq & 1) * 512 + l16 * 16;

#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < steps) issue(s, s);

  for (int step = 0; step < steps; ++step) {
    // stage `step` has landed once at most (S - 2) later stages of this wave are still in flight
    if (step + S - 2 < steps) wait_vmcnt<(S - 2) * P::kLoads>(); else wait_vmcnt<0>();
    // Plain s_barrier: __syncthreads() would add a fence that drains vmcnt to 0 and with it the pipeline.
    // Each wave has waited for its own share of the stage above; LDS reads below are issued after the
    // barrier in program order, and the compiler barriers keep them there.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();     // every wave's share of the stage is visible; the stage computed last step is free
    asm volatile("" ::: "memory");
    if (step + S - 1 < steps) issue((step + S - 1) % S, step + S - 1);

    const unsigned char* sa = smem_raw + (step % S) * P::kStage;
    const unsigned char* sb = sa + P::kAStage;
#pragma unroll
    for (int kk = 0; kk < BK / 32; ++kk) {
      half8 fa[2 * TM], fb[2 * TN];
      // the reads return in order: the first row of products can start after two of them
      fa[0] = *reinterpret_cast<const half8*>(sa + a_off[0] + (((4 * kk + kq) ^ a_swz[0]) * 16));
#pragma unroll
      for (int j = 0; j < 2 * TN; ++j)
        fb[j] = *reinterpret_cast<const half8*>(sb + ((wn * TN + (j >> 1)) * (BK / 16) + 2 * kk) * 1024 + (j & 1) * 256 + b_lane);
#pragma unroll
      for (int i = 1; i < 2 * TM; ++i)
        fa[i] = *reinterpret_cast<const half8*>(sa + a_off[i] + (((4 * kk + kq) ^ a_swz[i]) * 16));
#pragma unroll
      for (int i = 0; i < 2 * TM; ++i)
#pragma unroll
        for (int j = 0; j < 2 * TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue: every 32 x 32 accumulator tile goes through a private 32 x 33 fp32 patch of LDS
  // (lane = column on the way in, 8 consecutive columns of one row on the way out), so that the
  // epilogue functor stores runs of 8 columns instead of single elements.
  __syncthreads();                       // all waves have finished reading the last stage
  constexpr int kPitch = 36;             // floats: the four row groups of a sub-tile land 16 banks apart
  float* patch = reinterpret_cast<float*>(smem_raw) + wave * (32 * kPitch);
  static_assert(P::kLdsBytes >= P::kWaves * 32 * kPitch * 4, "the stage ring must hold one patch per wave");
  // Interior tiles (the vast majority) take a copy of the epilogue without bounds checks: with the per-store
  // branches gone the compiler can count the outstanding loads and stores exactly, instead of draining them
  // at every join.
  auto run_epilogue = [&](auto checked_tag) {
    constexpr bool kChecked = decltype(checked_tag)::value;
    half8 pre[epi_has_load<Epi>::value ? TN * TM * 2 : 1];
    if constexpr (epi_has_load<Epi>::value) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const int row = m0 + wm * 32 * TM + i * 32 + t * 16 + (lane >> 2), col = n0 + wn * 32 * TN + j * 32 + (lane & 3) * 8;
            half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            if (!kChecked || (row < M && col < N)) z = epi.load8(row, col);
            pre[(j * TM + i) * 2 + t] = z;
          }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int colbase = n0 + wn * 32 * TN + j * 32;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        // sub-tile (si, sj) of the 32 x 32 block: lane holds column 16 sj + l % 16 of rows 16 si + 4 (l / 16) + v
#pragma unroll
        for (int si = 0; si < 2; ++si)
#pragma unroll
          for (int sj = 0; sj < 2; ++sj)
#pragma unroll
            for (int v = 0; v < 4; ++v)
              patch[(si * 16 + 4 * kq + v) * kPitch + sj * 16 + l16] = acc[2 * i + si][2 * j + sj][v] + bvv[2 * j + sj];
        // same-wave LDS traffic: the compiler's lgkmcnt waits order the reads after the writes
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int r = t * 16 + (lane >> 2), c8 = (lane & 3) * 8;
          float o[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) o[q] = patch[r * kPitch + c8 + q];
          const int row = m0 + wm * 32 * TM + i * 32 + r, col = colbase + c8;
          if (!kChecked || (row < M && col < N)) {
            if constexpr (epi_has_load<Epi>::value) epi.store8(row, col, o, pre[(j * TM + i) * 2 + t]);
            else epi.store8(row, col, o);
          }
        }
      }
    }
  };
  if (m0 + P::kBM <= M && n0 + P::kBN <= N) run_epilogue(std::false_type{});
  else run_epilogue(std::true_type{});
}

}  // namespace ernie

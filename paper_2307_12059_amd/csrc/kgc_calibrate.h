// Calibration loops for the roofline of kernel 2 (gfx950): what the matrix pipes of this chip sustain on bf16 data
// of the join's kind, and what feeding them costs.  Every loop issues v_mfma_f32_32x32x16_bf16 on a wave tile of
// TM x TN accumulator blocks, as the join kernels do, on pseudo-random bf16 operands of unit scale, for long enough
// (hundreds of milliseconds) that the clock the chip settles on under that load is the one measured.
//
//   feed 0   operands stay in registers: the matrix pipes alone
//   feed 1   the TM head fragments of every K step are read from LDS (ds_read_b128), as in the join kernels
//   feed 2   ... and the TN tail fragments are read from global memory through the vector cache, in the join
//            kernel's access pattern (16 bytes per lane, a slice of 64-byte rows per two K steps, a range of rows
//            small enough to stay in the L2), two slices ahead of their use
// Wave tiles: 4 x 2 blocks (128 accumulator registers, two waves per SIMD, the join kernels' shape) and 4 x 4
// blocks (256 accumulator registers, one wave per SIMD).
#pragma once
#include <type_traits>

#include "kgc_device.h"

namespace kgc {

struct CalibArgs {
  const uint16_t* G;      // tail rows: [slices][rows][32] bf16, `rows` a multiple of 256
  int64_t rows;
  int slices;
  int iters;              // K steps per wave (a multiple of 2 * slices)
  float* sink;            // never written in practice; keeps the accumulators alive
};

__device__ __forceinline__ uint16_t calib_bf16(uint32_t i) {
  // sign, exponent 124 .. 127 (0.125 .. 1.99), 7 mantissa bits, from an integer hash
  uint32_t h = i * 2654435761u;
  h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
  return (uint16_t)((h & 0x8000u) | ((124u + ((h >> 8) & 3u)) << 7) | (h & 0x7fu));
}

__global__ void k_calib_fill(uint16_t* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = calib_bf16((uint32_t)i);
}

template <int I, int N, typename F>
__device__ __forceinline__ void calib_static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    calib_static_for<I + 1, N>(f);
  }
}

// WGM x WGN waves; the block's head tile is WGM * TM * 32 rows, kept in LDS for `KSL` slices
template <int TM, int TN, int WGM, int WGN, int FEED>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void k_calib_mfma(const CalibArgs a) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
  constexpr int KSL = 4;                                   // head slices in LDS (the loop walks them round and round)
  constexpr int ASZ = BM * 32;
  __shared__ __attribute__((aligned(16))) uint16_t lds[KSL * ASZ];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  for (int i = tid; i < KSL * ASZ; i += NT) lds[i] = calib_bf16((uint32_t)(i + blockIdx.x * 7919));
  __syncthreads();
  const int rsw = (((lane >> 2) & 1) << 1) | (((lane >> 1) ^ (lane >> 3)) & 1);
  const uint16_t* rd0 = lds + (wm * TM * 32 + (lane & 31)) * 32 + (((lane >> 5) ^ rsw) * 8);
  const uint16_t* rd1 = rd0 + ((((lane >> 5) ^ rsw) & 2) ? -16 : 16);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  bf16x8_t fa[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(rd0 + i * 1024);

  typedef uint32_t regq_t __attribute__((ext_vector_type(8 * TN)));
  regq_t q[3];
  // tail rows of this wave: the block's BN-row tile walks over the rows of the buffer, tile after tile
  const int64_t slice_bytes = a.rows * 64;
  const uint32_t voffB = (uint32_t)((wn * TN * 32 + (lane & 31)) * 64 + (lane >> 5) * 16);
  const int ntiles = (int)(a.rows / BN);
  int tile = (int)((blockIdx.x * 5u) % (unsigned)ntiles), sl = 0;
  const char* pB = (const char*)a.G + (int64_t)tile * BN * 64;
#define KGC_CAL_GLOAD(Q)                                                                          \
  do {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                              \
      const uint4 t0 = *(const uint4*)(pB + (voffB + (uint32_t)(j * 2048)));                      \
      const uint4 t1 = *(const uint4*)(pB + (voffB + (uint32_t)(j * 2048 + 32)));                 \
      Q[8 * j] = t0.x; Q[8 * j + 1] = t0.y; Q[8 * j + 2] = t0.z; Q[8 * j + 3] = t0.w;             \
      Q[8 * j + 4] = t1.x; Q[8 * j + 5] = t1.y; Q[8 * j + 6] = t1.z; Q[8 * j + 7] = t1.w;         \
    }                                                                                             \
    if (++sl == a.slices) {                                                                       \
      sl = 0;                                                                                     \
      tile = tile + 1 < ntiles ? tile + 1 : 0;                                                    \
      pB = (const char*)a.G + (int64_t)tile * BN * 64;                                            \
    } else {                                                                                      \
      pB += slice_bytes;                                                                          \
    }                                                                                             \
  } while (0)
#define KGC_CAL_FRAG(Q, J, STEP)                                                                  \
  __builtin_bit_cast(bf16x8_t, u32x4_t{Q[8 * (J) + 4 * (STEP)], Q[8 * (J) + 4 * (STEP) + 1],      \
                                       Q[8 * (J) + 4 * (STEP) + 2], Q[8 * (J) + 4 * (STEP) + 3]})
  if (FEED >= 2) {
    KGC_CAL_GLOAD(q[0]);
    KGC_CAL_GLOAD(q[1]);
  } else {
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
      for (int e = 0; e < 8 * TN; ++e) q[s][e] = (uint32_t)calib_bf16((uint32_t)(tid * 131 + s * 17 + e)) * 0x10001u;
  }

  // three slices (six K steps) per trip, so that the register sets of the tail prefetch are named statically
  for (int it = 0; it < a.iters; it += 6) {
    calib_static_for<0, 6>([&](auto S) __attribute__((always_inline)) {
      constexpr int s = decltype(S)::value;
      constexpr int set = s >> 1, half = s & 1;
      if constexpr (FEED >= 2 && half == 0) {
        KGC_CAL_GLOAD(q[(set + 2) % 3]);
        __builtin_amdgcn_sched_barrier(0);
      }
      constexpr int sn = (s + 1) % (2 * KSL);
      const uint16_t* An = ((sn & 1) ? rd1 : rd0) + (sn >> 1) * ASZ;
      calib_static_for<0, TM>([&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_CAL_FRAG(q[set], j, half), acc[i][j], 0, 0, 0);
        if constexpr (FEED >= 1) {
          fa[i] = *(const bf16x8_t*)(An + i * 1024);
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    });
  }
#undef KGC_CAL_GLOAD
#undef KGC_CAL_FRAG
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  if (s == 12345.678f) a.sink[blockIdx.x * NT + tid] = s;   // data-dependent and never true in practice
}

}  // namespace kgc

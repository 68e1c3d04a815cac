// Kernel 2, dense default: the barrier-free head-resident join with a straight-line tile body (gfx950, wave64).
//
// Same data flow as k_join_l2_direct (kgc_kernels.h): a block owns one (relation, head tile) and a range of
// tail tiles, keeps all K slices of its 256-row head tile in LDS, and every wave reads the MFMA fragments of its
// own 64 tail columns straight from the staged operand array, two slices ahead of their use through three
// register sets.  What differs is the instruction stream of a wave between its MFMAs, which is what bounds the
// matrix pipes once two waves share a SIMD:
//   * the number of 16-wide K steps is a template parameter, so a tile is straight-line code: no slice counters,
//     no data-dependent branches, every LDS address an immediate offset, the tail pointer a scalar;
//   * the head fragment of a block row for K step s + 1 is requested from LDS right behind the row's two MFMAs of
//     step s, into the registers they have just read (the order is pinned by scheduling barriers): one fragment
//     set, and six MFMAs for every LDS read to complete under;
//   * the head tile comes in by non-temporal loads (it is read once per block), so that the stream of head tiles
//     does not push the tail range out of the L2;
//   * the filter on a finished tile (minimum of the squared distances, Section 4.3's dist for p = 2 on the
//     bf16 operands) is folded into the FIRST K step of the next tile: block row by block row, the minimum of
//     two accumulator blocks is taken just ahead of the two MFMAs that overwrite them with a zero C operand, so
//     the vector work of the filter runs under the matrix work of the neighbouring blocks.  A block row that
//     holds a candidate records its element masks before it is overwritten; the exact path then runs once the
//     step's MFMAs are issued and re-issues them afterwards (its registers are the accumulators').  The exact path
//     is inlined: as a call it made every wave launch set up a stack, 6 us more per block.
// The minimum is taken on the float bits as signed integers: for a threshold >= 0, x <= thr holds exactly when
// bits(x) <= bits(thr) (negative x have negative bits), and an integer minimum needs no NaN canonicalisation.
// Three tiles are unrolled so that the three register sets of the tail prefetch are named statically.
#pragma once
#include <type_traits>

#include "kgc_kernels.h"

namespace kgc {

__device__ __forceinline__ int imin3(int a, int b, int c) { return min(min(a, b), c); }

// f(integral_constant<int, I>) for I = 0 .. N - 1, as straight-line code (no reliance on loop unrolling)
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// The exact path of a wave tile of 4 x 2 accumulator blocks.  Candidate masks: bit (16 * (2 * (i % 2) + j) + v) of
// word i / 2 is element v of block (i, j); MFMA 32x32 accumulator layout: register v of lane l holds row
// 8*(v/4) + 4*(l/32) + (v%4), column l%32.
__device__ __forceinline__ void dense_emit(unsigned long long cm0, unsigned long long cm1, int64_t hbase, int64_t tbase,
                                           int32_t r, const RecheckCtx& cx) {
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const unsigned long long cm = w == 0 ? cm0 : cm1;
    if (__builtin_amdgcn_ballot_w64(cm != 0ull) == 0ull) continue;
    recheck_and_emit(cm, r, cx, [=](int e, int src, int64_t& hslot, int64_t& tslot) {
      const int blk = w * 4 + (e >> 4), v = e & 15;
      const int i = blk >> 1, j = blk & 1;
      hslot = hbase + i * 32 + 8 * (v >> 2) + 4 * (src >> 5) + (v & 3);
      tslot = tbase + j * 32 + (src & 31);
    });
  }
}

template <int K16>
__global__ __launch_bounds__(512, 1) void k_join_l2_dense(const JoinStreamArgs a) {
  constexpr int NS = 3;                                   // register sets of the tail prefetch (NS - 1 slices ahead)
  constexpr int BM = 256, BN = 256, WGN = 4, NT = 512;
  constexpr int KS = (K16 + 1) / 2;                       // 32-wide slices; the last one holds one step when K16 is odd
  constexpr int TM = 4, TN = 2, WTM = 128, WTN = 64;
  constexpr int LA = (BM * 4) / NT;
  constexpr int ASZ = BM * kSliceK;
  constexpr int ROWB = kSliceK * 2;
  static_assert(K16 >= 1 && KS <= 9, "the head tile must fit in LDS");

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // [KS][BM][32] head slices
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // the same for the whole wave: scalar from here on
  const int wm = wave / WGN, wn = wave % WGN;
  const int tH = (int)blockIdx.x, rl = (int)blockIdx.y;
  const int t_begin = (int)(((int64_t)a.nT * blockIdx.z) / gridDim.z);
  const int t_end = (int)(((int64_t)a.nT * (blockIdx.z + 1)) / gridDim.z);
  const int ntiles = t_end - t_begin;
  if (ntiles <= 0) return;
  const int64_t slice_bytes = a.Nslots * ROWB;

  // fragment of K step `half` of a slice: logical 16-byte chunk 2 * half + lane / 32 of row lane % 32
  const int rsw = lds_swizzle(lane & 31);
  const uint16_t* rd0 = lds + (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const uint16_t* rd1 = rd0 + ((((lane >> 5) ^ rsw) & 2) ? -16 : 16);

  // tail fragments of this lane: row (lane % 32) of each 32-row group of the wave's columns; the tile / slice
  // part of the address is the same for the whole wave and stays in scalar registers
  const char* Bt = (const char*)a.B + (a.b_per_rel ? (int64_t)rl * KS * a.Nslots * ROWB : 0);
  const uint32_t voffB = (uint32_t)((wn * WTN + (lane & 31)) * ROWB + (lane >> 5) * 16);
  const char* pB = Bt + (int64_t)t_begin * BN * ROWB;     // slice being requested
  int pf_t = 0;                                            // its tile (stops on the last one: loads stay unconditional)

  typedef uint32_t regq_t __attribute__((ext_vector_type(8 * TN)));   // TN column groups x 2 K steps x 4 registers
  regq_t q[NS];
  // WRAP: the slice after this one is slice 0 of the next tile; BOTH: the slice holds two K steps of data
#define KGC_GLOAD(Q, WRAP, BOTH)                                                                  \
  do {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                              \
      const uint4 t0 = *(const uint4*)(pB + (voffB + (uint32_t)(j * 32 * ROWB)));                 \
      Q[8 * j] = t0.x; Q[8 * j + 1] = t0.y; Q[8 * j + 2] = t0.z; Q[8 * j + 3] = t0.w;             \
      if (BOTH) {                                                                                 \
        const uint4 t1 = *(const uint4*)(pB + (voffB + (uint32_t)(j * 32 * ROWB + 32)));          \
        Q[8 * j + 4] = t1.x; Q[8 * j + 5] = t1.y; Q[8 * j + 6] = t1.z; Q[8 * j + 7] = t1.w;       \
      }                                                                                           \
    }                                                                                             \
    if (WRAP) {                                                                                   \
      pf_t = pf_t + 1 < ntiles ? pf_t + 1 : pf_t;                                                 \
      pB = Bt + (int64_t)(t_begin + pf_t) * BN * ROWB;                                            \
    } else {                                                                                      \
      pB += slice_bytes;                                                                          \
    }                                                                                             \
  } while (0)
#define KGC_FRAG(Q, J, STEP)                                                                      \
  __builtin_bit_cast(bf16x8_t, u32x4_t{Q[8 * (J) + 4 * (STEP)], Q[8 * (J) + 4 * (STEP) + 1],      \
                                       Q[8 * (J) + 4 * (STEP) + 2], Q[8 * (J) + 4 * (STEP) + 3]})
#define KGC_LDA(F, KSL, HALF)                                                                     \
  do {                                                                                            \
    const uint16_t* Ac = ((HALF) ? rd1 : rd0) + (KSL) * ASZ;                                      \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) F[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK); \
  } while (0)
  // slice number `g` of the stream (counted from the tile the wave is in): which of its tile, and is it complete
#define KGC_SLICE_OF(g) ((g) % KS)
#define KGC_IS_LAST(g) (KGC_SLICE_OF(g) == KS - 1)
#define KGC_BOTH(g) (!KGC_IS_LAST(g) || (K16 % 2) == 0)

  // ---- head tile: all K slices into LDS, once (64-byte rows, 16-byte chunks XOR-swizzled by the row) ----
  {
    const char* Abase = (const char*)a.A + ((int64_t)rl * KS * a.Nslots + (int64_t)tH * BM) * ROWB;
    const uint32_t voff = (uint32_t)tid * 16u;
    const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
    constexpr int st_step = (NT / 4) * kSliceK;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 t[LA];
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        // read once per block and never again by this XCD: a non-temporal load, so that the stream of head tiles
        // does not push the tail range out of the L2
        const u32x4_t* src = (const u32x4_t*)(Abase + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));
        const u32x4_t v = __builtin_nontemporal_load(src);
        t[i] = make_uint4(v[0], v[1], v[2], v[3]);
      }
#pragma unroll
      for (int i = 0; i < LA; ++i) *(uint4*)(&lds[ks * ASZ + st0 + i * st_step]) = t[i];
    }
  }
  __syncthreads();          // the only barrier: the head tile is complete

  // (the threshold is the same for every lane: kept in a scalar register)
  const float thr = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.prm->thr)));
  const int thr_bits = thr >= 0.f ? __float_as_int(thr) : (int)0x80000000;   // negative threshold: nothing passes
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16;

  const int64_t hbase = (int64_t)tH * BM + wm * WTM;
  const int64_t tbase0 = (int64_t)t_begin * BN + wn * WTN;
  const int32_t rel = a.r0 + rl;
  const RecheckCtx cx = a.cx;

  int ct = 0;                                              // tiles finished
  bf16x8_t fa[TM];
  static_for<0, NS - 1>([&](auto G) __attribute__((always_inline)) {
    constexpr int g = decltype(G)::value;
    KGC_GLOAD(q[g], KGC_IS_LAST(g), KGC_BOTH(g));
  });
  KGC_LDA(fa, 0, 0);

  // one tile; U = its position in the group of three (which fixes the register sets of its slices).
  // Order inside a K step, pinned by scheduling barriers: (tail loads of the slice two ahead,) then per block row
  // its two MFMAs followed by the LDS read of the SAME row's fragment of the next step into the registers the two
  // MFMAs have just read -- one fragment set suffices, and every LDS read has six MFMAs to complete under.
  auto tile_body = [&](auto U) __attribute__((always_inline)) {
    constexpr int u = decltype(U)::value;
    static_for<0, K16>([&](auto S) __attribute__((always_inline)) {
      constexpr int s = decltype(S)::value;
      constexpr int ks = s >> 1, half = s & 1;
      constexpr int set = (u * KS + ks) % NS;
      if constexpr (half == 0) {
        KGC_GLOAD(q[(set + NS - 1) % NS], KGC_IS_LAST(ks + NS - 1), KGC_BOTH(ks + NS - 1));
        __builtin_amdgcn_sched_barrier(0);
      }
      constexpr int sn = (s + 1) % K16;
      const uint16_t* An = ((sn & 1) ? rd1 : rd0) + (sn >> 1) * ASZ;
      if constexpr (s == 0) {
        unsigned long long cm0 = 0ull, cm1 = 0ull;
        bool any = false;
        const int thr_now = ct > 0 ? thr_bits : (int)0x80000000;        // the first tile of a block follows none
        static_for<0, TM>([&](auto I) __attribute__((always_inline)) {
          constexpr int i = decltype(I)::value;
          int m = 0x7fffffff;
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; v += 2)
              m = imin3(m, __float_as_int(acc[i][j][v]), __float_as_int(acc[i][j][v + 1]));
          if (__builtin_amdgcn_ballot_w64(m <= thr_now) != 0ull) {
            unsigned long long bits = 0ull;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int v = 0; v < 16; ++v)
                if (__float_as_int(acc[i][j][v]) <= thr_now) bits |= 1ull << (16 * (2 * (i % 2) + j) + v);
            if (i < 2) cm0 |= bits; else cm1 |= bits;
            any = true;
          }
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_FRAG(q[set], j, 0), zero16, 0, 0, 0);
          fa[i] = *(const bf16x8_t*)(An + i * 32 * kSliceK);
          __builtin_amdgcn_sched_barrier(0);
        });
        if (any) {
          dense_emit(cm0, cm1, hbase, tbase0 + (int64_t)(ct - 1) * BN, rel, cx);
          // the exact path may take the accumulators' registers: the step is issued again
          bf16x8_t ft[TM];
          KGC_LDA(ft, 0, 0);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ft[i], KGC_FRAG(q[set], j, 0), zero16, 0, 0, 0);
        }
      } else {
        static_for<0, TM>([&](auto I) __attribute__((always_inline)) {
          constexpr int i = decltype(I)::value;
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_FRAG(q[set], j, half), acc[i][j], 0, 0, 0);
          fa[i] = *(const bf16x8_t*)(An + i * 32 * kSliceK);
          __builtin_amdgcn_sched_barrier(0);
        });
      }
    });
  };
  for (;;) {
    tile_body(std::integral_constant<int, 0>{});
    if (++ct == ntiles) break;
    tile_body(std::integral_constant<int, 1>{});
    if (++ct == ntiles) break;
    tile_body(std::integral_constant<int, 2>{});
    if (++ct == ntiles) break;
  }
  {   // the last tile of the range has no successor to hide its filter under
    int m = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; v += 2)
          m = imin3(m, __float_as_int(acc[i][j][v]), __float_as_int(acc[i][j][v + 1]));
    if (__builtin_amdgcn_ballot_w64(m <= thr_bits) != 0ull) {
      unsigned long long cm0 = 0ull, cm1 = 0ull;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (__float_as_int(acc[i][j][v]) <= thr_bits) {
              if (i < 2) cm0 |= 1ull << (16 * (2 * (i % 2) + j) + v);
              else cm1 |= 1ull << (16 * (2 * (i % 2) + j) + v);
            }
      dense_emit(cm0, cm1, hbase, tbase0 + (int64_t)(ct - 1) * BN, rel, cx);
    }
  }
#undef KGC_GLOAD
#undef KGC_FRAG
#undef KGC_LDA
#undef KGC_SLICE_OF
#undef KGC_IS_LAST
#undef KGC_BOTH
}

// the instantiation for a given number of K steps (1 .. 18)
typedef void (*dense_kernel_t)(const JoinStreamArgs);
template <int K>
struct DenseTable {
  static void fill(dense_kernel_t* t) {
    t[K] = k_join_l2_dense<K>;
    DenseTable<K - 1>::fill(t);
  }
};
template <>
struct DenseTable<0> {
  static void fill(dense_kernel_t*) {}
};
constexpr int kDenseMaxK16 = 18;
inline dense_kernel_t dense_kernel_for(int k16) {
  static dense_kernel_t table[kDenseMaxK16 + 1] = {};
  if (!table[1]) DenseTable<kDenseMaxK16>::fill(table);
  return (k16 >= 1 && k16 <= kDenseMaxK16) ? table[k16] : nullptr;
}

}  // namespace kgc

// Device-side helpers shared by the kernels of the TransE completion join (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kgc.h"

namespace kgc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// ---- bfloat16 <-> float32 (bf16 = upper half of an IEEE float32; round to nearest, ties to even) ----
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16_trunc(float x) { return (uint16_t)(__float_as_uint(x) >> 16); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// element `idx` of a float32 or bfloat16 array, widened to float (exact)
__device__ __forceinline__ float ld_elem(const void* base, int64_t idx, int dtype) {
  if (dtype == KGC_BF16) return bf16_to_f32(((const uint16_t*)base)[idx]);
  return ((const float*)base)[idx];
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }
// The same value, but opaque to the optimiser where it is taken: address arithmetic that the rare exact path derives
// from it then stays inside that path instead of being hoisted into (and spilled from) the kernel's prologue.
__device__ __forceinline__ int lane_id_here() {
  int l = (int)(threadIdx.x & 63u);
  asm volatile("" : "+v"(l));
  return l;
}

// ---- wave-level compaction (the "generate the results" step of Section 4.5) ----
// Every lane of the wave calls this with its own predicate.  One ballot gives the hit mask, its
// popcount the number of slots the wave needs, ONE atomic add by the first lane reserves them, and
// each hit lane's slot is the count of hit lanes below it.  Records beyond `cap` are dropped but
// still counted, so the counter ends at the true total.
__device__ __forceinline__ void wave_append(bool pred, int32_t h, int32_t r, int32_t t, float dist,
                                            kgc_triple* out, unsigned long long cap,
                                            unsigned long long* counter) {
  const unsigned long long m = __builtin_amdgcn_ballot_w64(pred);
  if (m == 0ull) return;
  const int n = __builtin_popcountll(m);
  const int lane = lane_id();
  const int first = __builtin_ctzll(m);
  unsigned long long base = 0ull;
  if (lane == first) base = atomicAdd(counter, (unsigned long long)n);
  const uint32_t blo = (uint32_t)__shfl((int)(uint32_t)(base & 0xffffffffull), first);
  const uint32_t bhi = (uint32_t)__shfl((int)(uint32_t)(base >> 32), first);
  base = ((unsigned long long)bhi << 32) | blo;
  const unsigned rank =
      __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
  if (pred) {
    const unsigned long long pos = base + rank;
    if (pos < cap) {
      kgc_triple rec;
      rec.h = h; rec.r = r; rec.t = t; rec.dist = dist;
      out[pos] = rec;
    }
  }
}

// What the second stage needs to re-score a candidate from the caller's arrays.
struct RecheckCtx {
  const void* E;             // rows of the head side: x = (E[h] + Rv[r]) - Et[t]
  const void* Et;            // rows of the tail side (the same array as E for the TransE join)
  const void* Rv;
  int64_t hstride, tstride;  // elements between the head / tail rows of consecutive relations: 0 for the TransE join
                             // (one entity array), N * d for per-relation connector outputs
  int64_t rstride;           // elements between relation vectors: d, or 0 when every relation reads row 0 of Rv
                             // (the general form, whose head rows already are connector_1(h, r): Rv is a zero row)
  const int32_t* slot_ent;   // slot -> entity row, -1 for padding (head side)
  const int32_t* slot_ent_t; // the same for the tail side (a join over a window of tiles counts its slots from the window's start)
  int dtype;
  int d;
  int p;
  double delta;
  kgc_triple* out;
  unsigned long long cap;
  unsigned long long* hit_counter;
  unsigned long long* cand_counter;
  int no_self;               // 1: candidates with h == t are dropped (the top-1 search without self pairs)
  // alignment of the caller's arrays, decided on the host (bases, d and strides), never found out on the device:
  int base16;                // 1: E, Et and Rv start on 16-byte boundaries (the 16-byte row reads of the per-candidate form
                             //    also need d % 4 == 0 for float32, d % 8 == 0 for bfloat16)
  int vec_ok;                // 1: every row starts on a boundary of four elements (16 bytes float32, 8 bytes bfloat16)
};

// Exact score of one triple by a 16-lane group (the TransE distance of Section 4.3 in double):
// x_k = (E[h][k] + Rv[r][k]) - E[t][k], s = sum x_k^2 or |x_k|, tree-reduced over the group; every lane of
// the group returns the norm.  When the rows are 16-byte aligned (d % 4 == 0 for float32, d % 8 == 0 for
// bfloat16) each lane reads 16-byte chunks, so that a candidate costs a couple of memory round trips
// rather than one per dimension.
__device__ __forceinline__ double group16_exact_dist(const RecheckCtx& cx, int32_t h, int32_t r, int32_t t, int sub) {
  const int d = cx.d;
  const int64_t ho = (int64_t)r * cx.hstride + (int64_t)h * d, to = (int64_t)r * cx.tstride + (int64_t)t * d,
                ro = (int64_t)r * cx.rstride;
  double s0 = 0.0, s1 = 0.0;
  const bool p2 = cx.p == 2;
  if (cx.dtype == KGC_F32 && (d & 3) == 0 && cx.base16) {
    const float4* eh = (const float4*)((const float*)cx.E + ho);
    const float4* et = (const float4*)((const float*)cx.Et + to);
    const float4* rv = (const float4*)((const float*)cx.Rv + ro);
    const int nch = d >> 2;
#pragma unroll 1
    for (int c = sub; c < nch; c += 16) {
      const float4 a0 = eh[c], b0 = rv[c], t0 = et[c];
      const double x0 = ((double)a0.x + (double)b0.x) - (double)t0.x, x1 = ((double)a0.y + (double)b0.y) - (double)t0.y;
      const double x2 = ((double)a0.z + (double)b0.z) - (double)t0.z, x3 = ((double)a0.w + (double)b0.w) - (double)t0.w;
      s0 += p2 ? (x0 * x0 + x1 * x1) : (fabs(x0) + fabs(x1));
      s1 += p2 ? (x2 * x2 + x3 * x3) : (fabs(x2) + fabs(x3));
    }
  } else if (cx.dtype == KGC_BF16 && (d & 7) == 0 && cx.base16) {
    const uint4* eh = (const uint4*)((const uint16_t*)cx.E + ho);
    const uint4* et = (const uint4*)((const uint16_t*)cx.Et + to);
    const uint4* rv = (const uint4*)((const uint16_t*)cx.Rv + ro);
    const int nch = d >> 3;
#pragma unroll 1
    for (int c = sub; c < nch; c += 16) {
      const uint4 a = eh[c], b = rv[c], tt = et[c];
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w}, tw[4] = {tt.x, tt.y, tt.z, tt.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const double xl = ((double)__uint_as_float(aw[q] << 16) + (double)__uint_as_float(bw[q] << 16)) -
                          (double)__uint_as_float(tw[q] << 16);
        const double xh = ((double)__uint_as_float(aw[q] & 0xffff0000u) + (double)__uint_as_float(bw[q] & 0xffff0000u)) -
                          (double)__uint_as_float(tw[q] & 0xffff0000u);
        s0 += p2 ? xl * xl : fabs(xl);
        s1 += p2 ? xh * xh : fabs(xh);
      }
    }
  } else {
#pragma unroll 1
    for (int k = sub; k < d; k += 16) {
      const double x = ((double)ld_elem(cx.E, ho + k, cx.dtype) + (double)ld_elem(cx.Rv, ro + k, cx.dtype)) -
                       (double)ld_elem(cx.Et, to + k, cx.dtype);
      s0 += p2 ? x * x : fabs(x);
    }
  }
  double s = s0 + s1;
  s += __shfl_xor(s, 8, 16);
  s += __shfl_xor(s, 4, 16);
  s += __shfl_xor(s, 2, 16);
  s += __shfl_xor(s, 1, 16);
  return p2 ? sqrt(s) : s;
}

// NC candidates of one relation at once (same arithmetic per candidate as group16_exact_dist): the loads of
// all of them are requested before any is used, so a drain step of the block-cooperative second stage pays
// one memory round trip per 16 x 4 (float32) or 16 x 8 (bfloat16) dimensions for NC candidates.  A negative
// h or t marks an absent candidate (its result is unused).
template <int NC>
__device__ __forceinline__ void group16_exact_dist_multi(const RecheckCtx& cx, const int32_t (&h)[NC], const int32_t (&t)[NC],
                                                         int32_t r, int sub, double (&out)[NC]) {
  const int d = cx.d;
  const bool p2 = cx.p == 2;
  const int64_t ro = (int64_t)r * cx.rstride;
  int64_t ho[NC], to[NC];
  double s0[NC], s1[NC];                 // two partial sums per candidate, as in the single form
#pragma unroll
  for (int n = 0; n < NC; ++n) {
    const bool ok = h[n] >= 0 && t[n] >= 0;      // an absent candidate reads row 0 and its result is ignored
    ho[n] = (int64_t)r * cx.hstride + (int64_t)(ok ? h[n] : 0) * d;
    to[n] = (int64_t)r * cx.tstride + (int64_t)(ok ? t[n] : 0) * d;
    s0[n] = 0.0; s1[n] = 0.0;
  }
  if (cx.dtype == KGC_F32 && (d & 3) == 0 && cx.base16) {
    const float4* rv = (const float4*)((const float*)cx.Rv + ro);
    const int nch = d >> 2;
#pragma unroll 1
    for (int c = sub; c < nch; c += 16) {
      const float4 rr = rv[c];
      float4 x[NC], y[NC];
#pragma unroll
      for (int n = 0; n < NC; ++n) {
        x[n] = ((const float4*)((const float*)cx.E + ho[n]))[c];
        y[n] = ((const float4*)((const float*)cx.Et + to[n]))[c];
      }
#pragma unroll
      for (int n = 0; n < NC; ++n) {
        const double q0 = ((double)x[n].x + (double)rr.x) - (double)y[n].x, q1 = ((double)x[n].y + (double)rr.y) - (double)y[n].y;
        const double q2 = ((double)x[n].z + (double)rr.z) - (double)y[n].z, q3 = ((double)x[n].w + (double)rr.w) - (double)y[n].w;
        s0[n] += p2 ? (q0 * q0 + q1 * q1) : (fabs(q0) + fabs(q1));
        s1[n] += p2 ? (q2 * q2 + q3 * q3) : (fabs(q2) + fabs(q3));
      }
    }
  } else if (cx.dtype == KGC_BF16 && (d & 7) == 0 && cx.base16) {
    const uint4* rv = (const uint4*)((const uint16_t*)cx.Rv + ro);
    const int nch = d >> 3;
#pragma unroll 1
    for (int c = sub; c < nch; c += 16) {
      const uint4 rr = rv[c];
      uint4 x[NC], y[NC];
#pragma unroll
      for (int n = 0; n < NC; ++n) {
        x[n] = ((const uint4*)((const uint16_t*)cx.E + ho[n]))[c];
        y[n] = ((const uint4*)((const uint16_t*)cx.Et + to[n]))[c];
      }
      const uint32_t rw[4] = {rr.x, rr.y, rr.z, rr.w};
#pragma unroll
      for (int n = 0; n < NC; ++n) {
        const uint32_t xw[4] = {x[n].x, x[n].y, x[n].z, x[n].w}, yw[4] = {y[n].x, y[n].y, y[n].z, y[n].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const double xl = ((double)__uint_as_float(xw[q] << 16) + (double)__uint_as_float(rw[q] << 16)) -
                            (double)__uint_as_float(yw[q] << 16);
          const double xh = ((double)__uint_as_float(xw[q] & 0xffff0000u) + (double)__uint_as_float(rw[q] & 0xffff0000u)) -
                            (double)__uint_as_float(yw[q] & 0xffff0000u);
          s0[n] += p2 ? xl * xl : fabs(xl);
          s1[n] += p2 ? xh * xh : fabs(xh);
        }
      }
    }
  } else {
#pragma unroll
    for (int n = 0; n < NC; ++n) out[n] = (h[n] >= 0 && t[n] >= 0) ? group16_exact_dist(cx, h[n], r, t[n], sub) : 0.0;
    return;
  }
#pragma unroll
  for (int n = 0; n < NC; ++n) {
    double s = s0[n] + s1[n];
    s += __shfl_xor(s, 8, 16);
    s += __shfl_xor(s, 4, 16);
    s += __shfl_xor(s, 2, 16);
    s += __shfl_xor(s, 1, 16);
    out[n] = p2 ? sqrt(s) : s;
  }
}

// ---- second stage, block form (L2): one 32 x 32 accumulator block re-scored by its wave on the fp64 matrix pipes ----
// Filter candidates come in patches: a pair of entity groups that a relation aligns fills much of a 32 x 32
// accumulator block, and re-scoring its pairs one by one reads every row dozens of times.  Here the wave that owns
// the block scores ALL its 1,024 pairs at once in double precision: a = (double)E[h] + (double)Rv[r] (exact) and
// t = (double)Et[t] are the operands of v_mfma_f64_16x16x4_f64, four dimensions per step, four 16 x 16 sub-blocks;
// the squared norms are summed beside it, and ||a - t||^2 = ||a||^2 + ||t||^2 - 2 a.t (the expansion of Section
// 4.3's dist for p = 2, now in double: with ||a||^2 + ||t||^2 of the order of d and an unit roundoff of 2^-53 its
// error is of the order of d^2 2^-53, some 1e-12 of the norms).  A pair is a hit when that value is below delta^2
// by more than this error, not a hit when it is above by more than it, and in the (practically empty) band between,
// or when a hit's value is tiny against the norms, the lane falls back to the definition: x_k = (E[h][k] + Rv[r][k]) - Et[t][k] in double, summed over k ascending,
// sqrt, <= delta.  Every true hit of the block passed the low-precision filter, so testing all pairs of the block
// gives exactly the hits among its candidates.  Hits leave with one reservation per block (a wave prefix sum over the
// lanes' hit counts), which the caller may share between waves.
//   hs0  slot of the block's first head row;  ts0  slot of its first tail column.   All 64 lanes call this together.
// Operand layout of the instruction: A[i][k] in lane 16 k + i, B[k][j] in lane 16 k + j, D[i][j] in element i / 4 of
// lane 16 (i % 4) + j (for double precision the four elements of a lane are four rows apart, not adjacent).
// It runs in a kernel of its own (k_exact_blocks) over the blocks the pruned join kernels LIST: inside the tile loop
// it either made the loop spill (inlined) or made every wave launch set up a stack (as a call), and a wave scoring
// a block held up the seven others of its tile; listed, the blocks of a whole launch are scored side by side.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
struct ExactEntry { int32_t r, hs0, ts0, pad; };             // relation, first head slot, first tail slot of a block
// four consecutive elements k .. k + 3 of a row, widened to float, zeros past d.  VEC: the row starts on a boundary of
// four elements and d is a multiple of four (one 16- or 8-byte load); otherwise element by element.
template <bool BF16, bool VEC>
__device__ __forceinline__ f32x4_t exact_ld4(const void* base, int64_t off, int k, int d) {
  f32x4_t o = {0.f, 0.f, 0.f, 0.f};
  if (VEC) {
    const int kc = k < d ? k : 0;                      // (past the end: a valid address, the values are dropped)
    if (BF16) {
      const uint2 v = *(const uint2*)((const uint16_t*)base + off + kc);
      o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
      o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    } else {
      const float4 v = *(const float4*)((const float*)base + off + kc);
      o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    if (k >= d) o = f32x4_t{0.f, 0.f, 0.f, 0.f};
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int ke = k + e < d ? k + e : 0;
      const float x = BF16 ? bf16_to_f32(((const uint16_t*)base)[off + ke]) : ((const float*)base)[off + ke];
      o[e] = k + e < d ? x : 0.f;
    }
  }
  return o;
}
// BF16: the storage type of the rows; VEC: rows may be read four elements at a time (template parameters, so that
// the loads below are straight-line code)
// reserve(total): called once by all lanes of the wave, returns the output position of the wave's first hit; the caller
// decides how waves share the atomic on the hit counter (thousands of atomics on one address cost more than the scoring).
template <bool BF16, bool VEC, typename Reserve>
__device__ __forceinline__ void exact_block_l2(int32_t r, const RecheckCtx& cx, int64_t hs0, int64_t ts0, Reserve reserve) {
  const int lane = lane_id_here();
  const int rr = lane & 15, kk = lane >> 4;         // operand row (or column), and which of a step's four operand slots
  const int d = cx.d, dtype = cx.dtype;
  int32_t hent[2], tent[2];
  int64_t ho[2], to[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    hent[q] = cx.slot_ent[hs0 + 16 * q + rr];
    tent[q] = cx.slot_ent_t[ts0 + 16 * q + rr];
    ho[q] = (int64_t)r * cx.hstride + (int64_t)(hent[q] < 0 ? 0 : hent[q]) * d;
    to[q] = (int64_t)r * cx.tstride + (int64_t)(tent[q] < 0 ? 0 : tent[q]) * d;
  }
  const int64_t ro = (int64_t)r * cx.rstride;
  f64x4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};
  double na[2] = {0.0, 0.0}, nt[2] = {0.0, 0.0};
  // A dot product does not care in which order its dimensions are taken as long as both operands agree, so the four
  // operand slots of a step need not hold four CONSECUTIVE dimensions: the dimensions are taken in groups of 16, and
  // lane (row, slot) reads the four consecutive elements 16 g + 4 slot .. + 3 of its row in one load and feeds them
  // to four successive steps (step e of the group multiplies dimensions 16 g + 4 slot + e, slot = 0 .. 3).
  // The rows are walked in chunks of kGroups groups: ALL loads of a chunk are issued before any is used, so a chunk
  // costs one memory round trip.  Elements past d count as zero.
  constexpr int kGroups = 2;
  for (int k0 = 0; k0 < d; k0 += 16 * kGroups) {
    f32x4_t hv[2][kGroups], tv[2][kGroups], rv[kGroups];
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
      const int k = k0 + 16 * g + 4 * kk;
      rv[g] = exact_ld4<BF16, VEC>(cx.Rv, ro, k, d);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        hv[q][g] = exact_ld4<BF16, VEC>(cx.E, ho[q], k, d);
        tv[q][g] = exact_ld4<BF16, VEC>(cx.Et, to[q], k, d);
      }
    }
    __builtin_amdgcn_sched_barrier(0);                 // (the loads stay together, ahead of the arithmetic)
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
      if (k0 + 16 * g >= d) break;                     // the same for the whole wave
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double av[2], bv[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          av[q] = (double)hv[q][g][e] + (double)rv[g][e];     // (elements past d were read as zeros)
          bv[q] = (double)tv[q][g][e];
          na[q] += av[q] * av[q];
          nt[q] += bv[q] * bv[q];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[i], bv[j], acc[i][j], 0, 0, 0);
      }
    }
  }
  // a row's norm: the sum over the four lanes that hold its operand slots 0 .. 3
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    na[q] += __shfl_xor(na[q], 16, 64); na[q] += __shfl_xor(na[q], 32, 64);
    nt[q] += __shfl_xor(nt[q], 16, 64); nt[q] += __shfl_xor(nt[q], 32, 64);
  }
  const double d2 = cx.delta * cx.delta;
  uint32_t hit = 0u;
  float dist[16];
  int32_t hsel[16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int hrow = 4 * v + kk;                   // the pair's head row inside sub-block row i: held by lane hrow
      const double nah = __shfl(na[i], hrow, 64);
      const int32_t h = __shfl(hent[i], hrow, 64);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int e = (i * 2 + j) * 4 + v;
        const int32_t t = tent[j];
        const double scale = nah + nt[j];
        const double D = scale - 2.0 * acc[i][j][v];
        float dd = 0.f;                                // (reported in float32: no square root in double needed)
        bool ok = D <= d2;
        const bool valid = h >= 0 && t >= 0 && !(cx.no_self && h == t);
        // too close to call from the expansion, or so small against the norms that its square root would carry the
        // expansion's error into the reported distance (near-duplicate rows, self pairs under r = 0): the definition
        if (valid && (fabs(D - d2) <= 1e-11 * scale || (D <= d2 && D < 1e-6 * scale))) {
          double ssum = 0.0;
          const int64_t hoff = (int64_t)r * cx.hstride + (int64_t)h * d, toff = (int64_t)r * cx.tstride + (int64_t)t * d;
          for (int k = 0; k < d; ++k) {
            const double x = ((double)ld_elem(cx.E, hoff + k, dtype) + (double)ld_elem(cx.Rv, ro + k, dtype)) -
                             (double)ld_elem(cx.Et, toff + k, dtype);
            ssum += x * x;
          }
          const double ds = sqrt(ssum);
          ok = ds <= cx.delta;
          dd = (float)ds;
        } else if (valid && ok) {
          dd = sqrtf((float)(D > 0.0 ? D : 0.0));
        }
        hsel[e] = h;
        dist[e] = dd;
        if (valid && ok) hit |= 1u << e;
      }
    }
  const int nh = __builtin_popcount(hit);
  int incl = nh;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off, 64);
    if (lane >= off) incl += o;
  }
  const int total = __shfl(incl, 63, 64);
  const unsigned long long base = reserve(total);
  if (total > 0) {
    unsigned long long pos = base + (unsigned long long)(incl - nh);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      if (!((hit >> e) & 1u)) continue;
      if (pos < cx.cap) {
        kgc_triple rec;
        rec.h = hsel[e]; rec.r = r; rec.t = tent[(e >> 2) & 1]; rec.dist = dist[e];
        cx.out[pos] = rec;
      }
      ++pos;
    }
  }
}

// ---- second stage: exact re-scoring of filter candidates + compaction ----
// `cm` holds, per lane, one bit for each of up to 64 accumulator elements of this lane that passed
// the low-precision filter.  `map(e, lane, hslot, tslot)` turns (element, owning lane) into the two
// slots.  Four candidates are re-scored at a time, one per 16-lane group: the group reads the three
// rows with consecutive lanes on consecutive dimensions, forms x = (E[h] + Rv[r]) - E[t] in double
// (the TransE distance of Section 4.3), sums x^2 or |x|, and tree-reduces over the group.  The
// decision dist <= delta is taken on that double.  All 64 lanes must call this together.
template <typename MapFn>
__device__ __forceinline__ void recheck_and_emit(unsigned long long cm, int32_t r, const RecheckCtx& cx,
                                                 MapFn map) {
  const int lane = lane_id_here();
  const int grp = lane >> 4, sub = lane & 15;
  unsigned long long ncand = 0ull;
  for (;;) {
    const unsigned long long b = __builtin_amdgcn_ballot_w64(cm != 0ull);
    if (b == 0ull) break;
    unsigned long long bb = b;
    for (int q = 0; q < grp; ++q) bb &= bb - 1ull;        // drop the grp lowest owners
    const int src = bb ? (int)__builtin_ctzll(bb) : -1;    // owner lane served by this group
    const int s2 = src < 0 ? lane : src;
    const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)(cm & 0xffffffffull), s2);
    const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)(cm >> 32), s2);
    const unsigned long long scm = ((unsigned long long)hi << 32) | lo;
    bool hit = false;
    float distf = 0.f;
    int32_t h = -1, t = -1;
    if (src >= 0) {
      const int e = (int)__builtin_ctzll(scm);
      int64_t hslot, tslot;
      map(e, src, hslot, tslot);
      h = cx.slot_ent[hslot];
      t = cx.slot_ent_t[tslot];
      if (h >= 0 && t >= 0 && !(cx.no_self && h == t)) {
        const double dist = group16_exact_dist(cx, h, r, t, sub);
        hit = dist <= cx.delta;
        distf = (float)dist;
      }
    }
    const int nb = __builtin_popcountll(b);
    ncand += (unsigned long long)(nb < 4 ? nb : 4);
    const int rank = __builtin_popcountll(b & ((1ull << lane) - 1ull));
    if (cm != 0ull && rank < 4) cm &= cm - 1ull;           // the four served owners retire one element
    wave_append(hit && sub == 0, h, r, t, distf, cx.out, cx.cap, cx.hit_counter);
  }
  if (lane == 0 && ncand) atomicAdd(cx.cand_counter, ncand);
}

// ---- block-cooperative form of the second stage ----
// Candidates of a tile cluster in one or two waves (an aligned pair of entity groups is a 32 x 32 patch),
// so re-scoring them inside the owning wave leaves the other waves idle.  Here every wave pushes its
// candidates into a small LDS queue and ALL 16-lane groups of the block drain it, four per wave at a time.
// The hits of a round are staged in LDS and leave with ONE global atomic per round: with a few hundred hits
// per tile, one atomic per wave step on the single output counter was what bounded the pruned join.
// Entered by the whole block together (the caller makes that decision block-uniform through q->flag).
template <int CAP>
struct BlockQueueT {
  static constexpr int kCap = CAP;
  unsigned int count;      // entries pushed in this round (may run past CAP: those pushes are retried)
  unsigned int pending;    // some wave still holds candidates after this round
  unsigned int flag;       // set by any wave whose tile has candidates; read after the block barrier
  unsigned int nhits;      // hits staged in this round
  unsigned long long base; // where this round's hits go in the output (one global atomic per round)
  unsigned long long ent[CAP];   // (hslot << 32) | tslot when pushed, then (head entity << 32) | tail entity (0xffffffff: padding row)
  kgc_triple hits[CAP];          // hits of this round, copied out together
};
using BlockQueue = BlockQueueT<512>;

// DRAIN: candidates per 16-lane group and drain step (their loads are in flight together); a kernel that is
// short of registers takes 1.
template <int NWAVES, int NW, int DRAIN, typename Queue, typename MapFn>
__device__ __forceinline__ void block_recheck(unsigned long long (&cm)[NW], int32_t r, const RecheckCtx& cx,
                                              Queue* q, MapFn map) {
  constexpr int kQueueCap = Queue::kCap;
  const int lane = lane_id();
  const int wave = (int)(threadIdx.x >> 6);
  const int grp = lane >> 4, sub = lane & 15;
  unsigned long long ncand = 0ull;
  for (;;) {
    // 1. every wave appends candidates (one per lane and pass) until its masks are empty or the queue is full
    for (int w = 0; w < NW; ++w) {
      for (;;) {
        const bool want = cm[w] != 0ull;
        const unsigned long long b = __builtin_amdgcn_ballot_w64(want);
        if (b == 0ull) break;
        const int n = __builtin_popcountll(b);
        const int first = __builtin_ctzll(b);
        unsigned int base = 0u;
        if (lane == first) base = atomicAdd(&q->count, (unsigned int)n);
        base = (unsigned int)__shfl((int)base, first);
        const unsigned rank =
            __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
        if (want && base + rank < (unsigned)kQueueCap) {
          const int e = (int)__builtin_ctzll(cm[w]);
          int64_t hslot, tslot;
          map(w * 64 + e, lane, hslot, tslot);
          q->ent[base + rank] = ((unsigned long long)(uint32_t)hslot << 32) | (unsigned long long)(uint32_t)tslot;
          cm[w] &= cm[w] - 1ull;
        }
        if (base + (unsigned)n >= (unsigned)kQueueCap) break;     // full: the rest waits for the next round
      }
    }
    bool more = false;
#pragma unroll
    for (int w = 0; w < NW; ++w) more |= cm[w] != 0ull;
    if (__builtin_amdgcn_ballot_w64(more) != 0ull && lane == 0) q->pending = 1u;
    __syncthreads();
    const unsigned int qn = q->count < (unsigned)kQueueCap ? q->count : (unsigned)kQueueCap;
    const unsigned int pend = q->pending;
    // 1b. slots -> entity numbers for the whole queue at once, one entry per thread, so that a drain step
    //     has one memory round trip (the rows) instead of two in a row; -1 (padding) becomes 0xffffffff
    for (unsigned int i = threadIdx.x; i < qn; i += NWAVES * 64) {
      const unsigned long long ent = q->ent[i];
      q->ent[i] = ((unsigned long long)(uint32_t)cx.slot_ent[(int64_t)(uint32_t)(ent >> 32)] << 32) |
                  (unsigned long long)(uint32_t)cx.slot_ent_t[(int64_t)(uint32_t)ent];
    }
    __syncthreads();
    // 2. all groups drain the queue, kDrain entries per group and step (entry e0 + 4 * wave + group and those
    //    NWAVES * 4 further), exact distance in double, hits staged in LDS
    constexpr int kDrain = DRAIN;
    for (unsigned int e0 = 0; e0 < qn; e0 += NWAVES * 4 * kDrain) {
      int32_t hh[kDrain], tt[kDrain];
      double dd[kDrain];
#pragma unroll
      for (int n = 0; n < kDrain; ++n) {
        const unsigned int e = e0 + (unsigned)(n * NWAVES * 4 + wave * 4 + grp);
        hh[n] = -1; tt[n] = -1;
        if (e < qn) {
          const unsigned long long ent = q->ent[e];
          hh[n] = (int32_t)(uint32_t)(ent >> 32);
          tt[n] = (int32_t)(uint32_t)ent;
          if (sub == 0) ++ncand;
        }
      }
      group16_exact_dist_multi<kDrain>(cx, hh, tt, r, sub, dd);
      if (sub == 0) {
#pragma unroll
        for (int n = 0; n < kDrain; ++n)
          if (hh[n] >= 0 && tt[n] >= 0 && !(cx.no_self && hh[n] == tt[n]) && dd[n] <= cx.delta) {
            kgc_triple rec;
            rec.h = hh[n]; rec.r = r; rec.t = tt[n]; rec.dist = (float)dd[n];
            q->hits[atomicAdd(&q->nhits, 1u)] = rec;         // LDS atomic; at most one hit per entry
          }
      }
    }
    __syncthreads();
    // 3. one global atomic reserves the output range of the whole round; all threads copy the hits out
    const unsigned int nh = q->nhits;
    if (threadIdx.x == 0 && nh) q->base = atomicAdd(cx.hit_counter, (unsigned long long)nh);
    __syncthreads();
    if (nh) {
      const unsigned long long base = q->base;
      for (unsigned int i = threadIdx.x; i < nh; i += NWAVES * 64) {
        const unsigned long long pos = base + i;
        if (pos < cx.cap) cx.out[pos] = q->hits[i];
      }
    }
    __syncthreads();
    if (threadIdx.x == 0) { q->count = 0u; q->pending = 0u; q->flag = 0u; q->nhits = 0u; }
    __syncthreads();
    if (!pend) break;
  }
  // per-wave candidate count (one lane per group counted its entries)
  for (int off = 32; off > 0; off >>= 1) ncand += __shfl_xor((unsigned long long)ncand, off, 64);
  if (lane == 0 && ncand) atomicAdd(cx.cand_counter, ncand);
}

}  // namespace kgc

// Device-side helpers shared by the kernels of the TransE completion join (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kgc.h"

namespace kgc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
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
  const void* E;
  const void* Rv;
  const int32_t* slot_ent;   // slot -> entity row, -1 for padding
  int dtype;
  int d;
  int p;
  double delta;
  kgc_triple* out;
  unsigned long long cap;
  unsigned long long* hit_counter;
  unsigned long long* cand_counter;
};

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
  const int lane = lane_id();
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
      t = cx.slot_ent[tslot];
      if (h >= 0 && t >= 0) {
        const int64_t ho = (int64_t)h * cx.d, to = (int64_t)t * cx.d, ro = (int64_t)r * cx.d;
        double s = 0.0;
        if (cx.p == 2) {
          for (int k = sub; k < cx.d; k += 16) {
            const double x = ((double)ld_elem(cx.E, ho + k, cx.dtype) + (double)ld_elem(cx.Rv, ro + k, cx.dtype)) -
                             (double)ld_elem(cx.E, to + k, cx.dtype);
            s += x * x;
          }
        } else {
          for (int k = sub; k < cx.d; k += 16) {
            const double x = ((double)ld_elem(cx.E, ho + k, cx.dtype) + (double)ld_elem(cx.Rv, ro + k, cx.dtype)) -
                             (double)ld_elem(cx.E, to + k, cx.dtype);
            s += fabs(x);
          }
        }
        s += __shfl_xor(s, 8, 16);
        s += __shfl_xor(s, 4, 16);
        s += __shfl_xor(s, 2, 16);
        s += __shfl_xor(s, 1, 16);
        const double dist = (cx.p == 2) ? sqrt(s) : s;
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

}  // namespace kgc

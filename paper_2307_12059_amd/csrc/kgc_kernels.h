// Kernels of the TransE completion join for gfx950 (CDNA4, wave64).
//
//   stage_operands   kernel 1: norms of the connector outputs (Section 4.3: a = h + r, b = t) with the zero
//                    vector as pivot (Section 4.5), and the bf16 operands of the contraction
//   join_l2          kernel 2: ||a - b||^2 for a tile of heads x tails by bf16 MFMA, filter, exact re-score
//   join_l1          kernel 3: sum |a - b| for a tile by float32 vector arithmetic, filter, exact re-score
// Both join kernels end in recheck_and_emit / wave_append (kgc_device.h).
#pragma once
#include "kgc_device.h"

namespace kgc {

// Number of extra contraction columns that carry the norms (three bf16 pieces of each float32 norm).
constexpr int kNormCols = 6;
// Operands are stored K-slice-major: X[ks][slot][32] bf16, so one tile's slice is contiguous.
constexpr int kSliceK = 32;
// Row stride (elements) of a slice in LDS: 32 + 8 padding = 80 bytes, which spreads eight consecutive
// rows' 16-byte fragments over all banks.
constexpr int kLdsRow = 40;
// Swizzle of the streaming kernel's LDS slices: rows are 64 bytes (four 16-byte chunks) without padding, and
// chunk c of row r is stored at position c ^ lds_swizzle(r).  With r = ...b3 b2 b1 b0 the swizzle is
// (b2 << 1) | (b1 ^ b3): eight or sixteen consecutive rows reading the same logical chunk, and four
// consecutive rows writing all their chunks, then fall on distinct banks whether the LDS serves 128 or
// 256 bytes per cycle.
__device__ __forceinline__ int lds_swizzle(int row) { return (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1); }
// Running maxima are kept in this many slots so that the atomics of kernel 1 do not pile on one address.
constexpr int kMaxSlots = 1024;

// device-side scalars of one join
struct JoinParams {
  float thr;            // filter threshold: on the squared distance (L2) or on the float32 sum (L1)
  float pad[3];
};

struct DevCounters {
  unsigned long long hits;        // true number of qualifying triples
  unsigned long long candidates;  // triples re-scored in double
  unsigned long long tile_cursor; // next free entry of the surviving-tile list (per relation batch)
  unsigned int n_active;          // rows (relation, head tile) of the batch that still have tail tiles
  unsigned int exact_need;        // most accumulator blocks any one batch wanted to list (see list_block)
  unsigned long long tiles;       // surviving tiles over all batches
  unsigned long long exact_total; // accumulator blocks scored by the block form of the exact stage, over all batches
  unsigned int max_a[1024];       // running maxima of ||bf16(h + r)||^2 (L2) or ||e||_1 (L1), float bits, spread over slots
  unsigned int max_b[1024];       // running maxima of ||bf16(t)||^2 (L2) or ||r||_1 (L1)
  unsigned int n_exact;           // accumulator blocks listed for the exact stage by the pruned L2 join kernels (per batch)
  unsigned int pair_mode;         // pruned L2 batch: 1 = its rows keep so few tiles that they are taken tile by tile
};

__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// relation numbers of a batch's records become numbers of the whole join (kgc_join_se)
__global__ void k_shift_relation(kgc_triple* rec, uint64_t n, int32_t r0) {
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) rec[i].r += r0;
}

// dense join over a window of head tiles: the (relation, 256-row tile) rows that the operand staging has to fill
__global__ void k_window_rows(uint32_t* rows, unsigned int* n_rows, int RB, int n_tiles, int w0, int w1) {
  const int per_rel = w1 - w0;
  const int64_t total = (int64_t)RB * per_rel;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
    rows[i] = (uint32_t)((i / per_rel) * n_tiles + w0 + i % per_rel);
  if (blockIdx.x == 0 && threadIdx.x == 0) *n_rows = (unsigned int)total;
}

// Around the tile lists of a pruned batch: the running total of surviving tiles, and which L2 join kernel takes the
// batch (when the host allows the choice): tile by tile when its rows keep few tiles.
//   phase 0, after k_rows_from_bitmap: at most kPairModeTilesPerRow tiles per active row on average.
//   phase 1, after a bound test that listed the new tiles itself (BoundL2Args::list_*) and before k_rows_from_bitmap:
//            the flat list is the batch's list when it is short against the number of rows (and fits); the rows then
//            count once per tile.  Otherwise the cursors start over and k_rows_from_bitmap builds the lists per row.
constexpr unsigned long long kPairModeTilesPerRow = 3;
__global__ void k_batch_tiles(DevCounters* c, int allow_pairs, int phase, unsigned long long n_rows, unsigned long long list_cap) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (phase == 0) {
      c->tiles += c->tile_cursor;
      c->pair_mode = (allow_pairs && c->tile_cursor <= kPairModeTilesPerRow * c->n_active && c->tile_cursor < 0xffffffffull) ? 1u : 0u;
    } else {
      const unsigned long long n = c->tile_cursor;
      const unsigned long long few = n_rows / 8 > 4096 ? n_rows / 8 : 4096;
      if (allow_pairs && n <= few && n <= list_cap && n < 0xffffffffull) {
        c->tiles += n; c->n_active = (unsigned int)n; c->pair_mode = 1u;
      } else {
        c->tile_cursor = 0; c->n_active = 0; c->pair_mode = 0u;
      }
    }
  }
}

// slot -> entity for the dense order: identity, -1 on the padding rows
__global__ void k_identity_slots(int32_t* slot_ent, int64_t N, int64_t Nslots) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < Nslots) slot_ent[i] = i < N ? (int32_t)i : -1;
}

// ---------------------------------------------------------------------------------------------
// Kernel 1.  One block stages kStageRows consecutive slots of one relation (IS_A: the row is
// a = h + r; otherwise the row is b = t and there is a single "relation").  The rows are rounded to bf16
// into an LDS tile, their squared norms ||.||^2 are summed in float32 from the rounded values, and the staged rows
//     A:  [ a~ (d) | nA_hi nA_mid nA_lo | 1 1 1 | 0 ... ]
//     B:  [ -2 b~ (d) | 1 1 1 | nB_hi nB_mid nB_lo | 0 ... ]
// are written slice by slice, 16 bytes per thread, so that the dot product of an A row and a B row is
// nA + nB - 2 a~.b~ = ||a~ - b~||^2.  The three pieces are the float32 norm cut into 8-bit mantissa
// chunks, exact in bf16.  Padding rows get a norm of 1e30 so they never pass the filter.  The squared
// norms are also written out plainly; with the zero pivot they are distA^2 and distB^2 of Section 4.5.
//
// Filter slack (slack_delta >= 0, the joins).  Rounding to bf16 moves a row x by e = ||x - x~||, which this
// kernel MEASURES per row (it holds x and x~) instead of bounding it by 2^-8 ||x||.  By the triangle
// inequality (the argument of Lemma 1, Section 4.4) a true hit ||a - b|| <= delta has
//     ||a~ - b~||^2 <= (delta + e_a + e_b)^2 <= delta^2 + (2 delta e_a + 2 e_a^2) + (2 delta e_b + 2 e_b^2),
// so each row's own term 2 delta e + 2 e^2 is taken off its norm column and the join compares against
// delta^2 (plus the float32 accumulation bound): rows that round well pay nothing for those that do not.
// e is widened by 0.1 % and by 2^-23 ||x|| (the float32 addition h + r and its own summation).
//
// Work split: a block of four waves stages kStageRows = 64 consecutive slots, 16 per wave, and nothing is shared
// between the waves (no block barrier).  A wave reads two rows per load instruction, 32 lanes x 4 consecutive
// dimensions each (one 16-byte or 8-byte load per lane where base and row length allow), keeps the per-row sums of
// squares in registers (8 row pairs), writes the rounded values to its own LDS tile, reduces the sums across lanes
// with a halving exchange (9 shuffles for 16 rows), adds the norm columns, and copies the tile out slice by slice,
// 1 KiB per store instruction.
constexpr int kStageRows = 64;
constexpr int kStageWaveRows = 16;

// four consecutive elements of a row from column c on (n = d - c of them exist); vec: 16-byte (f32) / 8-byte (bf16) loads allowed
__device__ __forceinline__ void stage_ld4(const void* base, int64_t off, int n, int dtype, bool vec, float v[4]) {
  v[0] = v[1] = v[2] = v[3] = 0.f;
  if (n <= 0) return;
  if (vec && n >= 4) {
    if (dtype == KGC_BF16) {
      const uint2 t = *(const uint2*)((const uint16_t*)base + off);
      v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
      v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    } else {
      const float4 t = *(const float4*)((const float*)base + off);
      v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    return;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k < n) v[k] = ld_elem(base, off + k, dtype);
}

// sums of 8 per-lane values over the 32 lanes of each half wave: afterwards lane l holds the total of value
// ((l >> 4) & 1) * 4 + ((l >> 3) & 1) * 2 + ((l >> 2) & 1)
__device__ __forceinline__ float stage_reduce8(const float v[8], int lane) {
  float a[4], b[2], c;
  const bool b4 = lane & 16, b3 = lane & 8, b2 = lane & 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float send = b4 ? v[i] : v[i + 4], keep = b4 ? v[i + 4] : v[i];
    a[i] = keep + __shfl_xor(send, 16, 64);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float send = b3 ? a[i] : a[i + 2], keep = b3 ? a[i + 2] : a[i];
    b[i] = keep + __shfl_xor(send, 8, 64);
  }
  {
    const float send = b2 ? b[0] : b[1], keep = b2 ? b[1] : b[0];
    c = keep + __shfl_xor(send, 4, 64);
  }
  c += __shfl_xor(c, 2, 64);
  c += __shfl_xor(c, 1, 64);
  return c;
}

template <bool IS_A>
__global__ __launch_bounds__(256, 4) void k_stage_operands(const void* __restrict__ E, const void* __restrict__ Rv,
                                                        int dtype, int d, int r0, int RB,
                                                        const int32_t* __restrict__ slot_ent, int64_t Nslots, int KS,
                                                        uint16_t* __restrict__ out, float* __restrict__ norms,
                                                        unsigned int* __restrict__ max_slots,
                                                        const uint32_t* __restrict__ active_rows,
                                                        const unsigned int* __restrict__ n_active, int nH, int bm,
                                                        int64_t rel_stride = 0, const int32_t* __restrict__ n_rows_dev = nullptr,
                                                        float slack_delta = -1.f,
                                                        int64_t n_identity = 0) {      // slot_ent == NULL: slot s holds entity s, s < n_identity
  extern __shared__ __attribute__((aligned(16))) uint16_t tile_all[];   // [4 waves][16 rows][KS * 32 + 8]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int W = KS * kSliceK + 8;
  uint16_t* tile = tile_all + wave * kStageWaveRows * W;
  const int esz = dtype == KGC_BF16 ? 2 : 4;
  // vector loads: every row of E (and of Rv) starts on a 4-element boundary of an aligned array
  const bool vec = (d % 4 == 0) && ((uintptr_t)E % (4 * esz) == 0) && (!(IS_A && Rv) || (uintptr_t)Rv % (4 * esz) == 0);
  const bool slack = slack_delta >= 0.f && slack_delta <= 3e38f;       // (an infinite threshold passes everything anyway)
  // dense joins stage every row group of every relation of the batch; pruned joins only the head tiles
  // (rows of the active list) that still have tail tiles to meet
  const int64_t groups_per_rel = Nslots / kStageRows;
  const int groups_per_tile = bm / kStageRows;
  const int64_t ngroups = active_rows ? (int64_t)*n_active * groups_per_tile : groups_per_rel * RB;
  float vmax = 0.f;
  for (int64_t g = blockIdx.x; g < ngroups; g += gridDim.x) {
    int rl;
    int64_t slot0;
    if (active_rows) {
      const int64_t row = (int64_t)active_rows[g / groups_per_tile];
      rl = (int)(row / nH);
      slot0 = (row - (int64_t)rl * nH) * bm + (g % groups_per_tile) * kStageRows;
    } else {
      rl = (int)(g / groups_per_rel);
      slot0 = (g - (int64_t)rl * groups_per_rel) * kStageRows;
    }
    // n_rows_dev: only the first *n_rows_dev slots (rounded up to a 256-row tile) hold rows this time
    if (n_rows_dev && slot0 >= ((int64_t)*n_rows_dev + 255) / 256 * 256) continue;
    slot0 += wave * kStageWaveRows;
    const int ent_l = lane >= kStageWaveRows ? -1 : slot_ent ? slot_ent[slot0 + lane] : (slot0 + lane < n_identity ? (int)(slot0 + lane) : -1);
    const int64_t ro = (int64_t)(r0 + rl) * d;
    const int64_t eo = (int64_t)(r0 + rl) * rel_stride;       // per-relation source rows (0: one array for all)
    float sq[8], er[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sq[i] = er[i] = 0.f;
    for (int c0 = 0; c0 < KS * kSliceK; c0 += 128) {
      const int c = c0 + 4 * l32;
      float rv[4] = {0.f, 0.f, 0.f, 0.f};
      if (IS_A && Rv) stage_ld4(Rv, ro + c, d - c, dtype, vec, rv);     // Rv == nullptr: the plain row (a = h)
      float x[8][4];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int ent = __shfl(ent_l, 2 * i + half, 64);
        stage_ld4(E, eo + (int64_t)(ent < 0 ? 0 : ent) * d + c, ent < 0 ? 0 : d - c, dtype, vec, x[i]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint16_t o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float v = x[i][k] + rv[k];                     // (columns past d and padding rows: 0 + 0)
          o[k] = f32_to_bf16_rne(v);
          const float f = bf16_to_f32(o[k]);
          sq[i] += f * f;
          er[i] += (v - f) * (v - f);
          if (!IS_A) o[k] = f32_to_bf16_rne(-2.f * f);        // B rows carry -2 b~ (exact: a sign flip and an exponent step)
        }
        if (c < KS * kSliceK)
          *(uint2*)(&tile[(2 * i + half) * W + c]) = make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
      }
    }
    // per-row totals: lane l now speaks for row 2 * i + half with i from bits 4, 3, 2 of l (four lanes hold the same)
    const float sqr = stage_reduce8(sq, lane), err = stage_reduce8(er, lane);
    {
      const int i = (((lane >> 4) & 1) << 2) | (((lane >> 3) & 1) << 1) | ((lane >> 2) & 1);
      const int row = 2 * i + half;
      const int ent_r = __shfl(ent_l, row, 64);
      float nrm = ent_r >= 0 ? sqr : 1e30f;
      const float plain = nrm;                                 // the maxima behind the accumulation bound stay plain
      if (slack && ent_r >= 0) {
        const float e = sqrtf(err) * 1.001f + 1.2e-7f * sqrtf(sqr);
        nrm = sqr - (2.f * slack_delta * e + 2.f * e * e) * 1.0001f;
      }
      if ((lane & 3) == 0) {
        uint16_t piece[3];
        float rem = nrm;
#pragma unroll
        for (int q = 0; q < 3; ++q) {
          piece[q] = f32_to_bf16_trunc(rem);
          rem -= bf16_to_f32(piece[q]);
        }
        const uint16_t one = 0x3F80u;
#pragma unroll
        for (int q = 0; q < kNormCols; ++q)
          tile[row * W + d + q] = (q < 3) == IS_A ? piece[q % 3] : one;
        if (norms) norms[(int64_t)rl * Nslots + slot0 + row] = plain;
        if (ent_r >= 0) vmax = fmaxf(vmax, plain);
      }
    }
    // the tile is this wave's own: its LDS operations complete in order, the fence keeps the compiler from moving them
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    {   // write out: slice ks of these 16 rows is 16 * 64 contiguous bytes
      const int row = lane >> 2, part = lane & 3;
      uint16_t* obase = out + ((int64_t)rl * KS * Nslots + slot0) * kSliceK + lane * 8;
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 v = *(const uint4*)(&tile[row * W + ks * kSliceK + part * 8]);
        *(uint4*)(obase + (int64_t)ks * Nslots * kSliceK) = v;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
  if (max_slots) {   // one atomic per wave, spread over kMaxSlots addresses
    for (int off = 32; off > 0; off >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, off, 64));
    if (lane == 0) atomicMax(&max_slots[(blockIdx.x * 4 + wave) % kMaxSlots], __float_as_uint(vmax));   // non-negative floats order like their bits
  }
}

// squared norms scattered back to entity order (kgc_norms)
__global__ void k_scatter_norms(const float* __restrict__ norms, const int32_t* __restrict__ slot_ent, int64_t Nslots,
                                int64_t N, int RB, float* __restrict__ outp) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)RB * Nslots) return;
  const int rl = (int)(i / Nslots);
  const int ent = slot_ent[i - (int64_t)rl * Nslots];
  if (ent >= 0) outp[(int64_t)rl * N + ent] = norms[i];
}

// max over rows of the L1 norm (used for the float32 error bound of the L1 filter)
__global__ __launch_bounds__(256) void k_row_l1_max(const void* __restrict__ X, int64_t rows, int d, int dtype,
                                                    unsigned int* __restrict__ max_bits) {
  const int j = threadIdx.x & 31;
  const int64_t hw = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 5;
  const int64_t nhw = ((int64_t)gridDim.x * blockDim.x) >> 5;
  float vmax = 0.f;
  for (int64_t row = hw; row < rows; row += nhw) {
    float s = 0.f;
    for (int c = j; c < d; c += 32) s += fabsf(ld_elem(X, row * d + c, dtype));
    s += __shfl_xor(s, 16, 32);
    s += __shfl_xor(s, 8, 32);
    s += __shfl_xor(s, 4, 32);
    s += __shfl_xor(s, 2, 32);
    s += __shfl_xor(s, 1, 32);
    vmax = fmaxf(vmax, s);
  }
  if (j == 0) atomicMax(&max_bits[blockIdx.x % kMaxSlots], __float_as_uint(vmax));
}

// Filter thresholds, computed on the device so that no host round trip sits between kernel 1 and the join.
//
// L2.  The staged norm columns already carry every row's own rounding slack (see k_stage_operands), so that a
// true hit has D' = ||a~ - b~||^2 - slack_a - slack_b <= delta^2.  The contraction returns D' with an accumulated
// float32 error of at most e_acc, so the filter keeps D' <= delta^2 + e_acc and loses no hit.
// L1.  The float32 sum of |fl(fl(h + r) - t)| differs from the exact sum by at most
// 2^-23 (max||h||_1 + max||r||_1) + (d + 2) 2^-23 (delta + that); the filter keeps sums below delta + margin.
__global__ __launch_bounds__(64) void k_join_params(DevCounters* cnt, JoinParams* prm, float delta, int p, int dtype,
                                                    int d, int kp) {
  float ma = 0.f, mb = 0.f;
  for (int i = threadIdx.x; i < 1024; i += 64) {
    ma = fmaxf(ma, __uint_as_float(cnt->max_a[i]));
    mb = fmaxf(mb, __uint_as_float(cnt->max_b[i]));
  }
  for (int off = 32; off > 0; off >>= 1) {
    ma = fmaxf(ma, __shfl_xor(ma, off, 64));
    mb = fmaxf(mb, __shfl_xor(mb, off, 64));
  }
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float thr;
  if (delta < 0.f) {
    thr = -1.f;                                   // squared distances and sums are >= 0: nothing passes
  } else if (p == 2) {
    const float eacc = (float)(kp + 16) * 1.2e-7f * 2.f * (ma + mb);
    thr = (delta * delta + eacc) * (1.f + 1e-6f);
  } else {
    const float base = 1.2e-7f * (ma + mb);
    thr = (delta + base + (float)(d + 2) * 1.2e-7f * (delta + base)) * (1.f + 1e-6f);
  }
  prm->thr = thr;
}

// ---------------------------------------------------------------------------------------------
struct JoinArgs {
  const uint16_t* A;        // staged A operands of this relation batch: [RB][KS][Nslots][32]   (L2)
  const uint16_t* B;        // staged B operands: [KS][Nslots][32]                              (L2)
  const JoinParams* prm;
  int64_t Nslots;
  int KS;                   // 32-wide slices
  int k16;                  // 16-wide MFMA steps that hold data (the last slice may be half empty)
  int nH, nT;               // tiles along heads / tails
  int r0, RB;               // first relation and number of relations of this batch
  RecheckCtx cx;
};

// Kernel 2.  One block scores one (relation, head tile, tail tile): D = A_tile * B_tile^T over the
// augmented K (Section 4.3's dist for p = 2, squared, on bf16-rounded operands), with bf16 MFMA
// 32x32x16 and float32 accumulation.  K slices go global -> registers -> LDS, double buffered.
// WGM x WGN waves; each wave owns a (BM/WGM) x (BN/WGN) sub-tile as TM x TN MFMA tiles.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(WGM* WGN * 64) void k_join_l2(const JoinArgs a) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LA = (BM * 4) / NT, LB = (BN * 4) / NT;   // 16-byte chunks per thread per slice
  static_assert(LA * NT == BM * 4 && LB * NT == BN * 4, "tile rows must divide over the threads");
  static_assert(TM >= 1 && TN >= 1, "wave tile too small");

  __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * kLdsRow];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * kLdsRow];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  const int tT = (int)blockIdx.x, tH = (int)blockIdx.y, rl = (int)blockIdx.z;

  const int64_t slice_elems = a.Nslots * kSliceK;
  const uint16_t* Ab = a.A + (int64_t)rl * a.KS * slice_elems + (int64_t)tH * BM * kSliceK;
  const uint16_t* Bb = a.B + (int64_t)tT * BN * kSliceK;

  uint4 ra[LA], rb[LB];
  auto gload = [&](int ks) {
    const uint4* ga = (const uint4*)(Ab + (int64_t)ks * slice_elems);
    const uint4* gb = (const uint4*)(Bb + (int64_t)ks * slice_elems);
#pragma unroll
    for (int i = 0; i < LA; ++i) ra[i] = ga[tid + i * NT];
#pragma unroll
    for (int i = 0; i < LB; ++i) rb[i] = gb[tid + i * NT];
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int c = tid + i * NT;
      *(uint4*)(&As[buf][(c >> 2) * kLdsRow + (c & 3) * 8]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      const int c = tid + i * NT;
      *(uint4*)(&Bs[buf][(c >> 2) * kLdsRow + (c & 3) * 8]) = rb[i];
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  gload(0);
  sstore(0);
  __syncthreads();

  const int arow = wm * WTM + (lane & 31);
  const int brow = wn * WTN + (lane & 31);
  const int koff = (lane >> 5) * 8;

  for (int ks = 0; ks < a.KS; ++ks) {
    const int buf = ks & 1;
    if (ks + 1 < a.KS) gload(ks + 1);
    const int steps = (a.k16 - ks * 2) >= 2 ? 2 : 1;
    for (int s = 0; s < steps; ++s) {
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *(const bf16x8_t*)(&As[buf][(arow + i * 32) * kLdsRow + s * 16 + koff]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *(const bf16x8_t*)(&Bs[buf][(brow + j * 32) * kLdsRow + s * 16 + koff]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (ks + 1 < a.KS) sstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: filter on the squared distance, then the rare exact path ----
  const float thr = a.prm->thr;
  float mn = acc[0][0][0];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) mn = fminf(mn, acc[i][j][v]);
  if (__builtin_amdgcn_ballot_w64(mn <= thr) == 0ull) return;

  // MFMA 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
  const int64_t hbase = (int64_t)tH * BM + wm * WTM;
  const int64_t tbase = (int64_t)tT * BN + wn * WTN;
  constexpr int NW = (TM * TN + 3) / 4;      // 64-element words of the candidate mask
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    unsigned long long cm = 0ull;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int tile = w * 4 + q;
      if (tile < TM * TN) {
        const int i = tile / TN, j = tile % TN;
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (acc[i][j][v] <= thr) cm |= 1ull << (q * 16 + v);
      }
    }
    if (__builtin_amdgcn_ballot_w64(cm != 0ull) == 0ull) continue;
    recheck_and_emit(cm, a.r0 + rl, a.cx, [&](int e, int src, int64_t& hslot, int64_t& tslot) {
      const int tile = w * 4 + (e >> 4), v = e & 15;
      const int i = tile / TN, j = tile % TN;
      hslot = hbase + i * 32 + 8 * (v >> 2) + 4 * (src >> 5) + (v & 3);
      tslot = tbase + j * 32 + (src & 31);
    });
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel 2, streaming form.  One block owns one (relation, head tile) and walks over a range of tail
// tiles; the K slices of all those tiles form one continuous stream that is prefetched two slices
// ahead through registers into a double-buffered LDS stage, so the global-memory latency of a slice
// is covered by the MFMA work of the two slices before it, also across tile boundaries.
// Tail-tile range: dense mode splits [0, nT) evenly over gridDim.z, the slowest grid dimension (x = head tile,
// y = relation), so that one range of tail rows stays in the L2 caches while every head tile of every
// relation passes over it; pruned mode reads the row's list of surviving tail tiles.
struct JoinStreamArgs {
  const uint16_t* A;
  const uint16_t* B;
  const JoinParams* prm;
  int64_t Nslots;
  int KS, k16;
  int nH, nT;
  int r0, RB;
  const uint32_t* row_start; // NULL: dense.  Else row = r_local * nH + head tile owns cols[row_start[row] .. + row_count[row])
  const uint32_t* row_count;
  const uint32_t* cols;      // surviving tail tile numbers, ascending within a row
  const uint32_t* active_rows;   // pruned mode: the rows with row_count > 0 ...
  const unsigned int* n_active;  // ... and how many there are; the grid strides over them
  RecheckCtx cx;
  ExactEntry* xlist;                  // where the kernel lists the accumulator blocks that hold candidates (k_exact_blocks
  unsigned int* xcount;               // scores them), how many it has listed, and how many the list holds; a block that
  unsigned int xcap;                  // finds the list full is counted, not stored (the host enlarges the list and reruns)
  const uint32_t* tile_rows;          // pruned mode, tile-at-a-time kernel: the row of every entry of cols ...
  const unsigned long long* tile_total;   // ... how many entries there are ...
  const unsigned int* pair_mode;      // ... and whether that kernel (1) or the row-walking one (0) takes this batch
  int cols_lds;                       // head-resident listed kernel: entries of LDS reserved for a row's tile list
  int b_per_rel;                      // 1: the tail operands are staged per relation, [RB][KS][Nslots][32] like A
  // Group assignment (k_join_l2_direct<.., kEpiAssignMin>): heads are all entities in identity order, tails
  // the pivots of a covering round, staged in an array of their own with tail_slots rows.
  int64_t tail_slots;                 // rows per K slice of B when it differs from Nslots (0: the same)
  const int32_t* tail_rows_dev;       // device count of valid tail rows (tail tiles past it are skipped); may be NULL
  float thr_value;                    // filter threshold on the squared distance when prm == NULL
  unsigned long long* best;           // kEpiAssignMin: per entity, min over the pivots within reach of (pivot position << 32);
                                      // kEpiMinDist: one word, min over all scored pairs of the float bits of the squared distance
  const int32_t* group_of;            // entities that already belong to a group (>= 0) are left alone
  int64_t n_heads;                    // entities (head slots past it are padding)
};
enum { kEpiJoin = 0, kEpiAssignMin = 1, kEpiMinDist = 2 };

// A 32 x 32 accumulator block with candidates, at the end of a tile: listed for k_exact_blocks.  A full list drops
// the entry but still counts it: the host then sees how long the list has to be and runs the join again.
__device__ __forceinline__ void list_block(const JoinStreamArgs& a, int32_t r, int64_t hs0, int64_t ts0) {
  if (lane_id() == 0) {
    const unsigned int idx = atomicAdd(a.xcount, 1u);
    if (idx < a.xcap) a.xlist[idx] = ExactEntry{r, (int32_t)hs0, (int32_t)ts0, 0};
  }
}

// The exact stage of the L2 joins that list blocks: one wave per listed block (exact_block_l2), the grid strides over
// the list.  Workgroups of kExactWaves waves: the waves of a workgroup score their blocks side by side and reserve
// their output records with ONE atomic on the hit counter between them (two barriers per round; the sums of a round
// sit in the LDS buffer of the round's parity, so a wave that is already in the next round does not overwrite what a
// slower one still reads).  One atomic per block was measured at 18 of the kernel's 46 microseconds on a list of
// 2,400 blocks: atomics on one address are served one after the other, 8 ns each.
constexpr int kExactWaves = 16;
template <bool BF16, bool VEC>
__global__ __launch_bounds__(kExactWaves * 64, 1) void k_exact_blocks(const ExactEntry* __restrict__ list, const unsigned int* __restrict__ count,
                                                      unsigned int cap, unsigned long long* __restrict__ total,
                                                      unsigned int* __restrict__ need, const RecheckCtx cx) {
  __shared__ unsigned int wave_hits[2][kExactWaves];
  __shared__ unsigned long long wave_base[2][kExactWaves];
  const unsigned int n = *count < cap ? *count : cap;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *total += n;
    if (*count > *need) *need = *count;
  }
  // entry e goes to wave e / gridDim.x of workgroup e % gridDim.x: a short list is spread over all workgroups (and with
  // them over all compute units), not over the waves of the first few
  const unsigned int wv = (unsigned int)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), per_round = gridDim.x * kExactWaves;
  int round = 0;
  for (unsigned int e0 = 0; e0 < n; e0 += per_round, ++round) {          // the same number of rounds for the whole workgroup
    const int par = round & 1;
    auto reserve = [&](int hits) -> unsigned long long {
      if ((threadIdx.x & 63) == 0) wave_hits[par][wv] = (unsigned int)hits;
      __syncthreads();
      if (threadIdx.x == 0) {
        unsigned int sum = 0u;
        for (int w = 0; w < kExactWaves; ++w) sum += wave_hits[par][w];
        unsigned long long base = sum ? atomicAdd(cx.hit_counter, (unsigned long long)sum) : 0ull;
        for (int w = 0; w < kExactWaves; ++w) { wave_base[par][w] = base; base += wave_hits[par][w]; }
      }
      __syncthreads();
      return wave_base[par][wv];
    };
    const unsigned int e = e0 + blockIdx.x + gridDim.x * wv;
    if (e < n) {                                                         // (the same for the whole wave)
      const ExactEntry x = list[e];
      exact_block_l2<BF16, VEC>(x.r, cx, (int64_t)x.hs0, (int64_t)x.ts0, reserve);
    } else {
      (void)reserve(0);
    }
  }
}

// LISTED: the block walks tile lists (pruned mode); otherwise the grid enumerates the dense problem and the
// kernel holds no load of the list in its inner loop (such a load would make every tile end wait for all
// outstanding prefetches).
template <int BM, int BN, int WGM, int WGN, int MINB, bool LISTED>
__global__ __launch_bounds__(WGM* WGN * 64, MINB) void k_join_l2_stream(const JoinStreamArgs a) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LA = (BM * 4) / NT, LB = (BN * 4) / NT;
  constexpr int ASZ = BM * kSliceK, BSZ = BN * kSliceK;      // elements per LDS buffer (64-byte rows, swizzled)
  static_assert(LA * NT == BM * 4 && LB * NT == BN * 4, "tile rows must divide over the threads");

  __shared__ __attribute__((aligned(16))) uint16_t As[2 * ASZ];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2 * BSZ];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  int ncand_lane = 0;                                        // candidates this lane sent to the exact stage

  // pruned mode: the grid strides over the rows (relation, head tile) that still have tail tiles
  for (unsigned int row_i = blockIdx.x;; row_i += gridDim.x) {
  int tH, rl, t_begin, t_end;
  const uint32_t* cols = nullptr;
  if constexpr (LISTED) {
    if (row_i >= *a.n_active) break;
    const int64_t row = (int64_t)a.active_rows[row_i];
    rl = (int)(row / a.nH); tH = (int)(row - (int64_t)rl * a.nH);
    t_begin = (int)a.row_start[row]; t_end = t_begin + (int)a.row_count[row];
    cols = a.cols;
    __syncthreads();                    // the previous row is done with the LDS buffers
  } else {
    // grid = (head tiles, tail-tile ranges, relations): blocks that run together share a tail-tile range
    tH = (int)blockIdx.x; rl = (int)blockIdx.y;
    t_begin = (int)(((int64_t)a.nT * blockIdx.z) / gridDim.z);
    t_end = (int)(((int64_t)a.nT * (blockIdx.z + 1)) / gridDim.z);
  }
  const int ntiles = t_end - t_begin;
  if (ntiles <= 0) break;
  const int KS = a.KS;
  const int64_t slice_bytes = a.Nslots * kSliceK * 2;

  // per-thread byte offset inside a tile slice; uniform bases are kept apart so they can live in SGPRs
  const uint32_t voff = (uint32_t)tid * 16u;
  const char* Abase = (const char*)a.A + ((int64_t)rl * KS * a.Nslots + (int64_t)tH * BM) * (kSliceK * 2);
  const char* Bbase = (const char*)a.B + (a.b_per_rel ? (int64_t)rl * KS * a.Nslots * (kSliceK * 2) : 0);
  int tcol = cols ? (int)cols[t_begin] : t_begin;
  const char* pA = Abase;                                            // slice being prefetched
  const char* pB = Bbase + (int64_t)tcol * BN * (kSliceK * 2);

  // LDS addresses (elements): where this thread stores its chunks (chunk i sits NT / 4 rows below chunk 0),
  // and where it reads its fragments
  const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
  constexpr int st_step = (NT / 4) * kSliceK;      // NT / 4 is a multiple of 16 rows, so the swizzle repeats
  // fragment of MFMA step s: logical 16-byte chunk 2 s + lane / 32 of row lane % 32; rows 32 apart share the swizzle
  const int rsw = lds_swizzle(lane & 31);
  const int rd_a = (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_b = (wn * WTN + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_step = (((lane >> 5) ^ rsw) & 2) ? -16 : 16;   // chunk ^ 2: the second step's fragment

  // staging registers as vectors (not arrays), so they are plain SSA values for the compiler
  typedef uint32_t rega_t __attribute__((ext_vector_type(4 * LA)));
  typedef uint32_t regb_t __attribute__((ext_vector_type(4 * LB)));
  rega_t ra;
  regb_t rb;

#define KGC_GLOAD()                                                                               \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < LA; ++i) {                                              \
      const uint4 t = *(const uint4*)(pA + voff + (uint32_t)(i * NT * 16));                       \
      ra[4 * i] = t.x; ra[4 * i + 1] = t.y; ra[4 * i + 2] = t.z; ra[4 * i + 3] = t.w;             \
    }                                                                                             \
    _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                              \
      const uint4 t = *(const uint4*)(pB + voff + (uint32_t)(i * NT * 16));                       \
      rb[4 * i] = t.x; rb[4 * i + 1] = t.y; rb[4 * i + 2] = t.z; rb[4 * i + 3] = t.w;             \
    }                                                                                             \
  } while (0)
#define KGC_SSTORE(AW, BW)                                                                        \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < LA; ++i)                                                \
      *(uint4*)(&(AW)[st0 + i * st_step]) = make_uint4(ra[4 * i], ra[4 * i + 1], ra[4 * i + 2], ra[4 * i + 3]); \
    _Pragma("unroll") for (int i = 0; i < LB; ++i)                                                \
      *(uint4*)(&(BW)[st0 + i * st_step]) = make_uint4(rb[4 * i], rb[4 * i + 1], rb[4 * i + 2], rb[4 * i + 3]); \
  } while (0)
#define KGC_MFMA_STEP(FA, FB)                                                                     \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
      _Pragma("unroll") for (int j = 0; j < TN; ++j)                                              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[i], FB[j], acc[i][j], 0, 0, 0);    \
  } while (0)

  // prologue: first slice -> registers -> LDS buffer 0
  KGC_GLOAD();
  KGC_SSTORE(As, Bs);
  __syncthreads();

  const float thr = a.prm->thr;
  const int last_two = (a.k16 - (KS - 1) * 2) >= 2;   // does the last slice of a tile hold two MFMA steps of data?
  int buf = 0;

  for (int ti = 0; ti < ntiles; ++ti) {
    f32x16_t acc[TM][TN];          // first written by the ks == 0 step, whose MFMAs take a zero C operand
    const int tcol_cur = tcol;

    for (int ks = 0; ks < KS; ++ks) {
      // ---- issue the loads of the next slice of the stream (next K slice, or slice 0 of the next tile) ----
      const bool last_slice = (ks == KS - 1);
      const bool has_next = !(last_slice && ti == ntiles - 1);
      if (has_next) {
        if (last_slice) {
          tcol = cols ? (int)cols[t_begin + ti + 1] : t_begin + ti + 1;
          pA = Abase;
          pB = Bbase + (int64_t)tcol * BN * (kSliceK * 2);
        } else {
          pA += slice_bytes;
          pB += slice_bytes;
        }
        KGC_GLOAD();
      }
      // ---- MFMA on the current slice ----
      const uint16_t* Ac = As + buf * ASZ + rd_a;
      const uint16_t* Bc = Bs + buf * BSZ + rd_b;
      {
        // all fragments of both MFMA steps are requested first, so the second step's LDS latency hides
        // behind the first step's MFMAs (the last slice of a tile may hold one step only)
        const bool two = !last_slice || last_two;
        bf16x8_t fa[TM], fb[TN], ga[TM], gb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *(const bf16x8_t*)(Bc + j * 32 * kSliceK);
        if (two) {
#pragma unroll
          for (int i = 0; i < TM; ++i) ga[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK + rd_step);
#pragma unroll
          for (int j = 0; j < TN; ++j) gb[j] = *(const bf16x8_t*)(Bc + j * 32 * kSliceK + rd_step);
        }
        if (ks == 0) {
          const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], zero16, 0, 0, 0);
        } else {
          KGC_MFMA_STEP(fa, fb);
        }
        if (two) KGC_MFMA_STEP(ga, gb);
      }
      // ---- stage the prefetched slice into the other buffer ----
      if (has_next) KGC_SSTORE(As + (buf ^ 1) * ASZ, Bs + (buf ^ 1) * BSZ);
      __syncthreads();
      buf ^= 1;
    }

    // ---- end of a tile: filter on the squared distance, then the rare exact path ----
    float mn = acc[0][0][0];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) mn = fminf(mn, acc[i][j][v]);
    const bool has = __builtin_amdgcn_ballot_w64(mn <= thr) != 0ull;
    // MFMA 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
    const int64_t hbase = (int64_t)tH * BM + wm * WTM;
    const int64_t tbase = (int64_t)tcol_cur * BN + wn * WTN;
    // Surviving tiles hold their candidates in patches: each accumulator block that has some is re-scored as a
    // whole in double precision by a kernel of its own: here it is only listed (list_block).
    if (has) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int n = 0;
#pragma unroll
          for (int v = 0; v < 16; ++v) n += (acc[i][j][v] <= thr) ? 1 : 0;
          if (__builtin_amdgcn_ballot_w64(n != 0) != 0ull) {
            ncand_lane += n;
            list_block(a, a.r0 + rl, hbase + i * 32, tbase + j * 32);
          }
        }
    }
  }
#undef KGC_GLOAD
#undef KGC_SSTORE
#undef KGC_MFMA_STEP
  if (!LISTED) break;
  }   // rows
  for (int off = 32; off > 0; off >>= 1) ncand_lane += __shfl_xor(ncand_lane, off, 64);
  if (lane == 0 && ncand_lane) atomicAdd(a.cx.cand_counter, (unsigned long long)ncand_lane);
}

// ---------------------------------------------------------------------------------------------
// Kernel 2, head-resident form.  As the streaming form, but the block first copies ALL K slices of its
// head tile (the staged a = h + r rows, BM x KS x 64 bytes) into LDS and keeps them there, so only the
// tail rows are streamed: half the global -> LDS traffic per tile, and the L2 only has to hold the tail
// range.  Tail slices are prefetched two slices ahead through two register sets.  Needs
// (KS * BM + 2 * BN) * 64 bytes of LDS: KS <= 8 (d <= 250) with one 256 x 256 block per CU, or with two 128 x 128 blocks per CU whose barriers and
// tile ends then fall at different times, so that one block's MFMAs fill the other's bubbles.
template <int BM, int BN, int WGM, int WGN, int MINB, int QCAP, bool LISTED>
__global__ __launch_bounds__(WGM* WGN * 64, MINB) void k_join_l2_ares(const JoinStreamArgs a) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LA = (BM * 4) / NT, LB = (BN * 4) / NT;
  constexpr int ASZ = BM * kSliceK, BSZ = BN * kSliceK;
  static_assert(LA * NT == BM * 4 && LB * NT == BN * 4, "tile rows must divide over the threads");

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // [KS][BM][32] head slices, then [2][BN][32] tail slices
  const int KS = a.KS;
  uint16_t* Ares = lds;
  uint16_t* Bs = lds + KS * ASZ;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  int ncand_lane = 0;                                        // candidates this lane sent to the exact stage
  if (LISTED && a.pair_mode && *a.pair_mode) return;         // this batch goes tile by tile (k_join_l2_pairs)

  for (unsigned int row_i = blockIdx.x;; row_i += gridDim.x) {
  int tH, rl, t_begin, t_end;
  const uint32_t* cols = nullptr;
  const uint32_t* lcols = nullptr;      // the row's tile list in LDS, when it fits (see below)
  if constexpr (LISTED) {
    if (row_i >= *a.n_active) break;
    const int64_t row = (int64_t)a.active_rows[row_i];
    rl = (int)(row / a.nH); tH = (int)(row - (int64_t)rl * a.nH);
    t_begin = (int)a.row_start[row]; t_end = t_begin + (int)a.row_count[row];
    cols = a.cols;
    __syncthreads();                    // the previous row is done with the LDS buffers
  } else {
    tH = (int)blockIdx.x; rl = (int)blockIdx.y;
    t_begin = (int)(((int64_t)a.nT * blockIdx.z) / gridDim.z);
    t_end = (int)(((int64_t)a.nT * (blockIdx.z + 1)) / gridDim.z);
  }
  const int ntiles = t_end - t_begin;
  if (ntiles <= 0) break;
  const int64_t slice_bytes = a.Nslots * kSliceK * 2;
  const uint32_t voff = (uint32_t)tid * 16u;
  const char* Abase = (const char*)a.A + ((int64_t)rl * KS * a.Nslots + (int64_t)tH * BM) * (kSliceK * 2);
  const char* Bbase = (const char*)a.B + (a.b_per_rel ? (int64_t)rl * KS * a.Nslots * (kSliceK * 2) : 0);
  int tcol = cols ? (int)cols[t_begin] : t_begin;
  const char* pB = Bbase + (int64_t)tcol * BN * (kSliceK * 2);

  const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
  constexpr int st_step = (NT / 4) * kSliceK;
  const int rsw = lds_swizzle(lane & 31);
  const int rd_a = (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_b = (wn * WTN + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_step = (((lane >> 5) ^ rsw) & 2) ? -16 : 16;

  // ---- head tile: all K slices into LDS, once; four slices' loads in flight together (a row with one or two
  // ---- tiles is mostly memory round trips); past the last slice the loads repeat it and nothing is stored
  for (int ks0 = 0; ks0 < KS; ks0 += 4) {
    uint4 t[4][LA];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ks = ks0 + j < KS ? ks0 + j : KS - 1;
#pragma unroll
      for (int i = 0; i < LA; ++i) t[j][i] = *(const uint4*)(Abase + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (ks0 + j < KS) {
#pragma unroll
        for (int i = 0; i < LA; ++i) *(uint4*)(&Ares[(ks0 + j) * ASZ + st0 + i * st_step]) = t[j][i];
      }
  }

  // The tile list of the row goes to LDS behind the tail buffers when there is room (a.cols_lds entries): the
  // loop then holds no global load besides the prefetches, whose outstanding count the compiler can follow
  // exactly; a list read from global memory makes every tile change wait for all of them.
  if (LISTED && ntiles <= a.cols_lds) {
    uint32_t* l = (uint32_t*)(Bs + 2 * BSZ);
    for (int t = tid; t < ntiles; t += NT) l[t] = cols[t_begin + t];
    lcols = l;
  }
  // the list must be complete before the first prefetches: with one or two K slices per tile they already move
  // on to the second tile (the barrier also publishes the head tile; all threads of a block take the same path)
  if (LISTED) __syncthreads();
  typedef uint32_t regb_t __attribute__((ext_vector_type(4 * LB)));
  regb_t rb0, rb1;
  int pf_k = 0, pf_t = 0, pf_i = 0;
#define KGC_GLOAD(RB)                                                                             \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < LB; ++i) {                                              \
      const uint4 t = *(const uint4*)(pB + voff + (uint32_t)(i * NT * 16));                       \
      RB[4 * i] = t.x; RB[4 * i + 1] = t.y; RB[4 * i + 2] = t.z; RB[4 * i + 3] = t.w;             \
    }                                                                                             \
    /* advance the cursor; past the end of the stream it stays on the last slice, so that the loads can be   */ \
    /* issued unconditionally (straight-line code lets the compiler count outstanding loads exactly)        */ \
    if (++pf_i < total) {                                                                         \
      if (++pf_k == KS) {                                                                         \
        pf_k = 0;                                                                                 \
        ++pf_t;                                                                                   \
        tcol = lcols ? (int)lcols[pf_t] : cols ? (int)cols[t_begin + pf_t] : t_begin + pf_t;          \
        pB = Bbase + (int64_t)tcol * BN * (kSliceK * 2);                                          \
      } else {                                                                                    \
        pB += slice_bytes;                                                                        \
      }                                                                                           \
    }                                                                                             \
  } while (0)
#define KGC_SSTORE(BUF, RB)                                                                       \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < LB; ++i)                                                \
      *(uint4*)(&Bs[(BUF) * BSZ + st0 + i * st_step]) =                                           \
          make_uint4(RB[4 * i], RB[4 * i + 1], RB[4 * i + 2], RB[4 * i + 3]);                     \
  } while (0)
#define KGC_MFMA_STEP(FA, FB)                                                                     \
  do {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
      _Pragma("unroll") for (int j = 0; j < TN; ++j)                                              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[i], FB[j], acc[i][j], 0, 0, 0);    \
  } while (0)

  const float thr = a.prm->thr;
  const int last_two = (a.k16 - (KS - 1) * 2) >= 2;
  const int total = ntiles * KS;
  int ck = 0, ct = 0;
  int tcol_cur = tcol;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // MFMA on tail slice in buffer BUF against head slice ck; at the end of a tile the filter on the squared
  // distance, the rare exact path, and the move to the next tile.  MFMA 32x32 accumulator layout: register v
  // of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
#define KGC_COMPUTE(BUF)                                                                          \
  do {                                                                                            \
    const uint16_t* Ac = Ares + ck * ASZ + rd_a;                                                  \
    const uint16_t* Bc = Bs + (BUF) * BSZ + rd_b;                                                 \
    const bool last_slice = (ck == KS - 1);                                                       \
    const bool two = !last_slice || last_two;                                                     \
    bf16x8_t fa[TM], fb[TN];                                                                      \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK); \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[j] = *(const bf16x8_t*)(Bc + j * 32 * kSliceK); \
    if (ck == 0) {                                                                                \
      const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], zero16, 0, 0, 0);     \
    } else {                                                                                      \
      KGC_MFMA_STEP(fa, fb);                                                                      \
    }                                                                                             \
    if (two) {                                                                                    \
      _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK + rd_step); \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[j] = *(const bf16x8_t*)(Bc + j * 32 * kSliceK + rd_step); \
      KGC_MFMA_STEP(fa, fb);                                                                      \
    }                                                                                             \
    if (last_slice) {                                                                             \
      /* End of a tile: does any element pass the filter?  Candidates come in patches, so every accumulator    */ \
      /* block that holds some is listed for the exact kernel (list_block): no queue, no extra barrier.         */ \
      /* MFMA 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32. */ \
      float mn = acc[0][0][0];                                                                    \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          _Pragma("unroll") for (int v = 0; v < 16; ++v) mn = fminf(mn, acc[i][j][v]);            \
      if (__builtin_amdgcn_ballot_w64(mn <= thr) != 0ull) {                                       \
        const int64_t hbase = (int64_t)tH * BM + wm * WTM;                                        \
        const int64_t tbase = (int64_t)tcol_cur * BN + wn * WTN;                                  \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                            \
          _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                        \
            int n = 0;                                                                            \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) n += (acc[i][j][v] <= thr) ? 1 : 0;    \
            if (__builtin_amdgcn_ballot_w64(n != 0) != 0ull) {                                    \
              ncand_lane += n;                                                                    \
              list_block(a, a.r0 + rl, hbase + i * 32, tbase + j * 32);                           \
            }                                                                                     \
          }                                                                                       \
      }                                                                                           \
      ck = 0;                                                                                     \
      if (++ct < ntiles) tcol_cur = lcols ? (int)lcols[ct] : cols ? (int)cols[t_begin + ct] : t_begin + ct; \
    } else {                                                                                      \
      ++ck;                                                                                       \
    }                                                                                             \
  } while (0)

  // prologue: tail slices 0 and 1 in flight, slice 0 staged (the barrier also publishes the head tile)
  KGC_GLOAD(rb0);
  KGC_GLOAD(rb1);
  KGC_SSTORE(0, rb0);
  __syncthreads();

  // Both steps run to their end in every iteration (an odd number of slices only skips the second step's
  // arithmetic): with no way out of the middle of the body, every path reaches the top of the loop with
  // the same loads outstanding, so the compiler needs no wait there.
  for (int i = 0; i < total; i += 2) {
    // even step: slice i is in buffer 0; set 0 is free for slice i + 2; set 1 holds slice i + 1
    KGC_GLOAD(rb0);
    KGC_COMPUTE(0);
    KGC_SSTORE(1, rb1);
    __syncthreads();
    // odd step: slice i + 1 is in buffer 1; set 1 is free for slice i + 3; set 0 holds slice i + 2
    KGC_GLOAD(rb1);
    if (i + 1 < total) KGC_COMPUTE(1);
    KGC_SSTORE(0, rb0);
    __syncthreads();
  }
#undef KGC_GLOAD
#undef KGC_SSTORE
#undef KGC_MFMA_STEP
#undef KGC_COMPUTE
  if (!LISTED) break;
  }   // rows
  for (int off = 32; off > 0; off >>= 1) ncand_lane += __shfl_xor(ncand_lane, off, 64);
  if (lane == 0 && ncand_lane) atomicAdd(a.cx.cand_counter, (unsigned long long)ncand_lane);
}

// ---------------------------------------------------------------------------------------------
// Kernel 2, one surviving tile at a time (pruned joins whose rows keep only a tile or two each).  Walking such a
// row costs the row-walking kernels a chain of some ten memory round trips (row record, tile list, head tile,
// the tail slices one behind the other) for a microsecond of arithmetic.  Here a block takes one (row, tail tile)
// entry of the list, reads ALL K slices of both 128-row tiles with every load in flight at once, and multiplies out
// of LDS: three round trips per tile.  The host launches both kernels; a device flag set from the batch's tile and
// row counts (k_batch_tiles) says which of them works.  LDS: 2 * KS * 8 KiB.
__global__ __launch_bounds__(256, 2) void k_join_l2_pairs(const JoinStreamArgs a) {
  constexpr int BM = 128, BN = 128, NT = 256, WGN = 2, WTM = 64, WTN = 64, TM = 2, TN = 2;
  constexpr int LA = (BM * 4) / NT;
  constexpr int ASZ = BM * kSliceK;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // [KS][128][32] head slices, then the same for the tail tile
  if (!*a.pair_mode) return;
  const int KS = a.KS;
  uint16_t* As = lds;
  uint16_t* Bs = lds + KS * ASZ;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const unsigned int total = (unsigned int)*a.tile_total;
  const int64_t slice_bytes = a.Nslots * kSliceK * 2;
  const uint32_t voff = (uint32_t)tid * 16u;
  const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
  constexpr int st_step = (NT / 4) * kSliceK;
  const int rsw = lds_swizzle(lane & 31);
  const int rd_a = (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_b = (wn * WTN + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_step = (((lane >> 5) ^ rsw) & 2) ? -16 : 16;
  const float thr = a.prm->thr;
  const bool last_two = (a.k16 - (KS - 1) * 2) >= 2;
  int ncand_lane = 0;
  // A block walks its tiles (entries blockIdx.x, + gridDim.x, ... of the list) in batches of up to kPairsBatch: the
  // batch's list entries are read into the LDS first, so that no load of the list sits among the tile loads (loads
  // return in order: waiting for a list entry would wait for every tile load asked for before it).  The first four K
  // slices of the NEXT tile are asked for as soon as the current tile is in the LDS, so that their memory round trip
  // runs beside the current tile's arithmetic.  Which of a tile's 32 x 32 blocks hold candidates is noted per wave,
  // and the batch's blocks are listed for the exact kernel at its end with ONE atomic on the list's length for the
  // whole workgroup (atomics on one address are served one after the other, and their round trip would sit in
  // every tile's path).
  constexpr int kPairsBatch = 32;
  __shared__ uint32_t my_row[kPairsBatch], my_col[kPairsBatch];
  __shared__ uint8_t my_has[kPairsBatch][4];
  __shared__ unsigned int list_n[4];
  __shared__ unsigned int list_base;
  typedef uint32_t regt_t __attribute__((ext_vector_type(16 * LA)));   // 4 slices x LA chunks x 4 registers: vectors, so
  regt_t ta, tb;                                                       // that they are plain SSA values for the compiler
#define KGC_PAIRS_ASK(ROW, TCOL)                                                                              \
  do {                                                                                                       \
    const int rl_ = (int)((ROW) / (uint32_t)a.nH), tH_ = (int)((ROW) - (uint32_t)rl_ * (uint32_t)a.nH);      \
    const char* Ab_ = (const char*)a.A + ((int64_t)rl_ * KS * a.Nslots + (int64_t)tH_ * BM) * (kSliceK * 2); \
    const char* Bb_ = (const char*)a.B + (a.b_per_rel ? (int64_t)rl_ * KS * a.Nslots * (kSliceK * 2) : 0) +  \
                      (int64_t)(TCOL) * BN * (kSliceK * 2);                                                  \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                          \
      const int ks = j < KS ? j : KS - 1; /* past the last slice the loads repeat it and nothing is stored */ \
      _Pragma("unroll") for (int i = 0; i < LA; ++i) {                                                       \
        const uint4 x_ = *(const uint4*)(Ab_ + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));  \
        const uint4 y_ = *(const uint4*)(Bb_ + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));  \
        ta[4 * (j * LA + i)] = x_.x; ta[4 * (j * LA + i) + 1] = x_.y; ta[4 * (j * LA + i) + 2] = x_.z; ta[4 * (j * LA + i) + 3] = x_.w; \
        tb[4 * (j * LA + i)] = y_.x; tb[4 * (j * LA + i) + 1] = y_.y; tb[4 * (j * LA + i) + 2] = y_.z; tb[4 * (j * LA + i) + 3] = y_.w; \
      }                                                                                                      \
    }                                                                                                        \
  } while (0)
  for (unsigned int e0 = blockIdx.x; e0 < total; e0 += kPairsBatch * gridDim.x) {      // (the same for the whole block)
    // the batch's entries e0, e0 + gridDim.x, ...
    const unsigned int left = (total - e0 + gridDim.x - 1) / gridDim.x;
    const int nb = left < (unsigned int)kPairsBatch ? (int)left : kPairsBatch;
    __syncthreads();                                         // the previous batch is listed
    if (tid < nb) { my_row[tid] = a.tile_rows[e0 + (unsigned int)tid * gridDim.x]; my_col[tid] = a.cols[e0 + (unsigned int)tid * gridDim.x]; }
    __syncthreads();
    KGC_PAIRS_ASK(my_row[0], my_col[0]);
    for (int it = 0; it < nb; ++it) {
    const uint32_t row = my_row[it], tcol_now = my_col[it];
    const int rl = (int)(row / (uint32_t)a.nH), tH = (int)(row - (uint32_t)rl * (uint32_t)a.nH);
    __syncthreads();                                         // the previous tile is done with the LDS
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (j < KS) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
          *(uint4*)(&As[j * ASZ + st0 + i * st_step]) = make_uint4(ta[4 * (j * LA + i)], ta[4 * (j * LA + i) + 1], ta[4 * (j * LA + i) + 2], ta[4 * (j * LA + i) + 3]);
          *(uint4*)(&Bs[j * ASZ + st0 + i * st_step]) = make_uint4(tb[4 * (j * LA + i)], tb[4 * (j * LA + i) + 1], tb[4 * (j * LA + i) + 2], tb[4 * (j * LA + i) + 3]);
        }
      }
    if (KS > 4) {                                            // the slices after the fourth: loaded now (d > 122)
      const char* Abase = (const char*)a.A + ((int64_t)rl * KS * a.Nslots + (int64_t)tH * BM) * (kSliceK * 2);
      const char* Bbase = (const char*)a.B + (a.b_per_rel ? (int64_t)rl * KS * a.Nslots * (kSliceK * 2) : 0) +
                          (int64_t)tcol_now * BN * (kSliceK * 2);
      for (int ks0 = 4; ks0 < KS; ks0 += 4) {
        uint4 ua[4][LA], ub[4][LA];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ks = ks0 + j < KS ? ks0 + j : KS - 1;
#pragma unroll
          for (int i = 0; i < LA; ++i) {
            ua[j][i] = *(const uint4*)(Abase + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));
            ub[j][i] = *(const uint4*)(Bbase + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (ks0 + j < KS) {
#pragma unroll
            for (int i = 0; i < LA; ++i) {
              *(uint4*)(&As[(ks0 + j) * ASZ + st0 + i * st_step]) = ua[j][i];
              *(uint4*)(&Bs[(ks0 + j) * ASZ + st0 + i * st_step]) = ub[j][i];
            }
          }
      }
    }
    __syncthreads();
    if (it + 1 < nb) KGC_PAIRS_ASK(my_row[it + 1], my_col[it + 1]);      // the next tile's loads
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int ks = 0; ks < KS; ++ks) {
      const uint16_t* Ac = As + ks * ASZ + rd_a;
      const uint16_t* Bc = Bs + ks * ASZ + rd_b;
      const int nstep = (ks < KS - 1 || last_two) ? 2 : 1;
      for (int step = 0; step < nstep; ++step) {
        bf16x8_t fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK + step * rd_step);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *(const bf16x8_t*)(Bc + j * 32 * kSliceK + step * rd_step);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
    }
    // the filter on the squared distance: which of the wave's blocks hold candidates
    unsigned int has = 0u;                                   // bit i * TN + j: block (i, j)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int n = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) n += (acc[i][j][v] <= thr) ? 1 : 0;
        ncand_lane += n;
        if (__builtin_amdgcn_ballot_w64(n != 0) != 0ull) has |= 1u << (i * TN + j);
      }
    if (lane == 0) my_has[it][wave] = (uint8_t)has;
    }   // tiles of the batch
    // the batch's blocks with candidates onto the list: wave w takes the notes of all four waves for tiles w, w + 4, ...
    __syncthreads();
    unsigned int mine = 0u;
    for (int it = wave; it < nb; it += 4)
      mine += (unsigned int)__builtin_popcount((unsigned int)my_has[it][0] | ((unsigned int)my_has[it][1] << 8) |
                                               ((unsigned int)my_has[it][2] << 16) | ((unsigned int)my_has[it][3] << 24));
    if (lane == 0) list_n[wave] = mine;
    __syncthreads();
    if (tid == 0) {
      const unsigned int sum = list_n[0] + list_n[1] + list_n[2] + list_n[3];
      list_base = sum ? atomicAdd(a.xcount, sum) : 0u;
    }
    __syncthreads();
    if (lane == 0 && mine) {
      unsigned int idx = list_base;
      for (int w = 0; w < wave; ++w) idx += list_n[w];
      for (int it = wave; it < nb; it += 4) {
        const uint32_t row = my_row[it];
        const int rl = (int)(row / (uint32_t)a.nH), tH = (int)(row - (uint32_t)rl * (uint32_t)a.nH);
        for (int w = 0; w < 4; ++w) {
          const unsigned int has = my_has[it][w];
          const int64_t hbase = (int64_t)tH * BM + (w / WGN) * WTM;
          const int64_t tbase = (int64_t)my_col[it] * BN + (w % WGN) * WTN;
          for (int b = 0; b < TM * TN; ++b)
            if ((has >> b) & 1u) {
              if (idx < a.xcap) a.xlist[idx] = ExactEntry{a.r0 + rl, (int32_t)(hbase + (b / TN) * 32), (int32_t)(tbase + (b % TN) * 32), 0};
              ++idx;
            }
        }
      }
    }
  }   // batches
#undef KGC_PAIRS_ASK
  for (int off = 32; off > 0; off >>= 1) ncand_lane += __shfl_xor(ncand_lane, off, 64);
  if (lane == 0 && ncand_lane) atomicAdd(a.cx.cand_counter, (unsigned long long)ncand_lane);
}

// ---------------------------------------------------------------------------------------------
// Kernel 2, barrier-free form (dense mode only).  The head tile is resident in LDS as above, but the tail
// rows never pass through LDS: every wave reads the MFMA fragments of ITS OWN WTN tail columns straight from
// the staged operand array into registers (lane l takes row l % 32 of a 32-row group, 16 bytes at offset
// 16 * (l / 32) for the first K step of a slice and 32 bytes further for the second: the layout the MFMA
// wants), two slices ahead of their use through three register sets.  Nothing in the loop is shared between
// waves, so it holds no barrier and no LDS store: the LDS only serves the head fragments, and the waves of
// a block drift apart, so that one wave's MFMAs cover the other's waits.  The waves that share tail columns
// (same wn) read the same lines, mostly one after the other out of the CU's vector cache.
// LDS: KS * BM * 64 bytes: BM = 256 up to KS = 9 (d <= 282), BM = 128 up to KS = 19 (d <= 602).  In the join
// form (EPI = kEpiJoin) candidates are re-scored by the owning wave; kEpiAssignMin is the epilogue of the
// group assignment (see JoinStreamArgs).
// LISTED (pruned joins over many entities, kEpiJoin): the grid strides over the active rows, and a row's tile list
// sits in the LDS behind the head slices (a.cols_lds entries), so that the tile loop holds no load of the list among
// its prefetches.
template <int BM, int WGM, int WGN, int EPI, bool LISTED = false>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void k_join_l2_direct(const JoinStreamArgs a) {
  constexpr int BN = 256;
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LA = (BM * 4) / NT;
  constexpr int ASZ = BM * kSliceK;
  constexpr int ROWB = kSliceK * 2;                       // bytes of one staged row slice
  static_assert(LA * NT == BM * 4, "tile rows must divide over the threads");

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // [KS][BM][32] head slices
  const int KS = a.KS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  for (unsigned int blk_i = blockIdx.x;; blk_i += gridDim.x) {
  unsigned int row_i = blk_i;
  int tH, rl, t_begin, ntiles;
  const uint32_t* tlist = nullptr;                         // LISTED: the row's tile list in the LDS
  if constexpr (LISTED) {
    // Workgroups go to the eight XCDs in turn, and neighbouring active rows (one relation, neighbouring head tiles)
    // meet the same tail tiles: within every 256 consecutive workgroups, those of one XCD take 32 neighbouring rows,
    // so that a tail tile is fetched into one L2, not into all eight.
    const unsigned int n_act = *a.n_active;
    if ((blk_i & ~255u) >= n_act) break;                   // (the same for the whole block)
    row_i = (blk_i & ~255u) + (blk_i & 7u) * 32u + ((blk_i >> 3) & 31u);
    if (row_i >= n_act) continue;                          // (a hole of the last, partial set of 256)
    // (the same for the whole block: kept in scalar registers)
    const int64_t row = (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)a.active_rows[row_i]);
    rl = (int)(row / a.nH); tH = (int)(row - (int64_t)rl * a.nH);
    t_begin = __builtin_amdgcn_readfirstlane((int)a.row_start[row]); ntiles = __builtin_amdgcn_readfirstlane((int)a.row_count[row]);
    __syncthreads();                                       // the previous row is done with the LDS
  } else {
    tH = (int)blockIdx.x; rl = (int)blockIdx.y;
    int nT = a.nT;
    if (EPI == kEpiAssignMin && a.tail_rows_dev) {        // only the tail tiles that hold pivots of this round
      const int used = (*a.tail_rows_dev + BN - 1) / BN;
      nT = used < nT ? used : nT;
    }
    t_begin = (int)(((int64_t)nT * blockIdx.z) / gridDim.z);
    ntiles = (int)(((int64_t)nT * (blockIdx.z + 1)) / gridDim.z) - t_begin;
  }
  if (ntiles <= 0) break;                                  // (an active row has tiles; the same for the whole block)
  const int64_t slice_bytes_a = a.Nslots * ROWB;
  const int64_t slice_bytes = (a.tail_slots ? a.tail_slots : a.Nslots) * ROWB;

  // ---- head tile: all K slices into LDS, once (swizzled as in the other forms) ----
  {
    const char* Abase = (const char*)a.A + ((int64_t)rl * KS * a.Nslots + (int64_t)tH * BM) * ROWB;
    const uint32_t voff = (uint32_t)tid * 16u;
    const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
    constexpr int st_step = (NT / 4) * kSliceK;
    for (int ks = 0; ks < KS; ++ks) {
      uint4 t[LA];
#pragma unroll
      for (int i = 0; i < LA; ++i) t[i] = *(const uint4*)(Abase + (int64_t)ks * slice_bytes_a + voff + (uint32_t)(i * NT * 16));
#pragma unroll
      for (int i = 0; i < LA; ++i) *(uint4*)(&lds[ks * ASZ + st0 + i * st_step]) = t[i];
    }
  }
  // LISTED: the row's tiles in segments of what the LDS holds of the list (a.cols_lds entries; nearly always one segment)
  const int row_tiles = ntiles;
  for (int seg0 = 0; seg0 < (LISTED ? row_tiles : 1); seg0 += (LISTED ? a.cols_lds : 1)) {
  if constexpr (LISTED) {
    if (seg0 > 0) __syncthreads();                         // the previous segment's list is no longer read
    ntiles = row_tiles - seg0 < a.cols_lds ? row_tiles - seg0 : a.cols_lds;
    uint32_t* l = (uint32_t*)(lds + KS * ASZ);
    for (int t = tid; t < ntiles; t += NT) l[t] = a.cols[t_begin + seg0 + t];
    tlist = l;
  }
  __syncthreads();          // the head tile (and the tile list) is complete: no barrier in the tile loop

  const int rsw = lds_swizzle(lane & 31);
  const int rd_a = (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_step = (((lane >> 5) ^ rsw) & 2) ? -16 : 16;

  // tail fragments of this lane: row (lane % 32) of each 32-row group of the wave's columns
  // (LISTED: the tile part of the address is the same for the whole wave and stays in scalar registers, the lane's
  // part is a 32-bit offset: the kernel has no register to spare)
  const uint32_t boff = (uint32_t)((wn * WTN + (lane & 31)) * ROWB + (lane >> 5) * 16);
  const char* Bw = (const char*)a.B + (a.b_per_rel ? (int64_t)rl * KS * a.Nslots * ROWB : 0) + (LISTED ? 0u : boff);
  const char* pB = Bw + (int64_t)(LISTED ? __builtin_amdgcn_readfirstlane((int)tlist[0]) : t_begin) * BN * ROWB;
  const int total = ntiles * KS;
  int pf_k = 0, pf_t = 0, pf_i = 0;

  typedef uint32_t regq_t __attribute__((ext_vector_type(8 * TN)));   // TN column groups x 2 K steps x 4 registers
  regq_t q0, q1, q2;
#define KGC_GLOAD(Q)                                                                              \
  do {                                                                                            \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                              \
      const uint4 t0 = *(const uint4*)(pB + ((LISTED ? boff : 0u) + (uint32_t)(j * 32 * ROWB)));  \
      const uint4 t1 = *(const uint4*)(pB + ((LISTED ? boff : 0u) + (uint32_t)(j * 32 * ROWB + 32))); \
      Q[8 * j] = t0.x; Q[8 * j + 1] = t0.y; Q[8 * j + 2] = t0.z; Q[8 * j + 3] = t0.w;             \
      Q[8 * j + 4] = t1.x; Q[8 * j + 5] = t1.y; Q[8 * j + 6] = t1.z; Q[8 * j + 7] = t1.w;         \
    }                                                                                             \
    /* the cursor stops on the last slice, so the loads are unconditional (and the compiler can count them) */ \
    if (++pf_i < total) {                                                                         \
      if (++pf_k == KS) {                                                                         \
        pf_k = 0;                                                                                 \
        ++pf_t;                                                                                   \
        pB = Bw + (int64_t)(LISTED ? __builtin_amdgcn_readfirstlane((int)tlist[pf_t]) : t_begin + pf_t) * BN * ROWB; \
      } else {                                                                                    \
        pB += slice_bytes;                                                                        \
      }                                                                                           \
    }                                                                                             \
  } while (0)
#define KGC_FRAG(Q, J, STEP)                                                                      \
  __builtin_bit_cast(bf16x8_t, u32x4_t{Q[8 * (J) + 4 * (STEP)], Q[8 * (J) + 4 * (STEP) + 1],      \
                                       Q[8 * (J) + 4 * (STEP) + 2], Q[8 * (J) + 4 * (STEP) + 3]})

  const float thr = a.prm ? a.prm->thr : a.thr_value;
  float run_min = 3e38f;                                   // kEpiMinDist
  const int last_two = (a.k16 - (KS - 1) * 2) >= 2;
  int ck = 0, ct = 0;
  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // One slice: head fragments from LDS, tail fragments from register set Q; at the end of a tile the filter
  // on the squared distance and the rare exact path.  MFMA 32x32 accumulator layout: register v of lane l
  // holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
#define KGC_COMPUTE(Q)                                                                            \
  do {                                                                                            \
    const uint16_t* Ac = lds + ck * ASZ + rd_a;                                                   \
    const bool last_slice = (ck == KS - 1);                                                       \
    const bool two = !last_slice || last_two;                                                     \
    bf16x8_t fa[TM];                                                                              \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK); \
    if (ck == 0) {                                                                                \
      const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_FRAG(Q, j, 0), zero16, 0, 0, 0); \
    } else {                                                                                      \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_FRAG(Q, j, 0), acc[i][j], 0, 0, 0); \
    }                                                                                             \
    if (two) {                                                                                    \
      _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK + rd_step); \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], KGC_FRAG(Q, j, 1), acc[i][j], 0, 0, 0); \
    }                                                                                             \
    if (last_slice) {                                                                             \
      float mn = acc[0][0][0];                                                                    \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
          _Pragma("unroll") for (int v = 0; v < 16; ++v) mn = fminf(mn, acc[i][j][v]);            \
      if (EPI == kEpiMinDist) {                                                                   \
        run_min = fminf(run_min, mn);        /* only the smallest squared distance is wanted */    \
      } else if (__builtin_amdgcn_ballot_w64(mn <= thr) != 0ull) {                                \
        const int64_t hbase = (int64_t)tH * BM + wm * WTM;                                        \
        const int64_t tbase = (int64_t)(LISTED ? __builtin_amdgcn_readfirstlane((int)tlist[ct]) : t_begin + ct) * BN + wn * WTN; \
        constexpr int NW = (TM * TN + 3) / 4;                                                     \
        _Pragma("unroll") for (int w = 0; w < NW; ++w) {                                          \
          unsigned long long cm = 0ull;                                                           \
          _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                         \
            const int tile = w * 4 + q;                                                           \
            if (tile < TM * TN) {                                                                 \
              const int i = tile / TN, j = tile % TN;                                             \
              _Pragma("unroll") for (int v = 0; v < 16; ++v)                                      \
                if (acc[i][j][v] <= thr) cm |= 1ull << (q * 16 + v);                              \
            }                                                                                     \
          }                                                                                       \
          if (__builtin_amdgcn_ballot_w64(cm != 0ull) == 0ull) continue;                          \
          auto map = [=](int e, int src, int64_t& hslot, int64_t& tslot) {                        \
            const int tile = w * 4 + (e >> 4), v = e & 15;                                        \
            const int i = tile / TN, j = tile % TN;                                               \
            hslot = hbase + i * 32 + 8 * (v >> 2) + 4 * (src >> 5) + (v & 3);                     \
            tslot = tbase + j * 32 + (src & 31);                                                  \
          };                                                                                      \
          if (EPI == kEpiJoin) {                                                                  \
            recheck_and_emit(cm, a.r0 + rl, a.cx, map);                                           \
          } else {                                                                                \
            /* every lane files its own elements; the lowest pivot position within reach wins (only the */ \
            /* position matters to the round: the low word, a distance in the float32 form, stays 0)   */ \
            while (cm) {                                                                          \
              const int e = (int)__builtin_ctzll(cm);                                             \
              cm &= cm - 1ull;                                                                    \
              int64_t hslot, tslot;                                                               \
              map(e, lane, hslot, tslot);                                                         \
              if (hslot < a.n_heads && a.group_of[hslot] < 0)                                     \
                atomicMin(&a.best[hslot], (unsigned long long)(uint32_t)tslot << 32);             \
            }                                                                                     \
          }                                                                                       \
        }                                                                                         \
      }                                                                                           \
      ck = 0;                                                                                     \
      ++ct;                                                                                       \
    } else {                                                                                      \
      ++ck;                                                                                       \
    }                                                                                             \
  } while (0)

  // slices i, i + 1 in flight; every step first asks for slice i + 2 (into the set slice i - 1 has left)
  KGC_GLOAD(q0);
  KGC_GLOAD(q1);
  for (int i = 0; i < total; i += 3) {
    KGC_GLOAD(q2);
    KGC_COMPUTE(q0);
    KGC_GLOAD(q0);
    if (i + 1 < total) KGC_COMPUTE(q1);
    KGC_GLOAD(q1);
    if (i + 2 < total) KGC_COMPUTE(q2);
  }
#undef KGC_GLOAD
#undef KGC_FRAG
#undef KGC_COMPUTE
  if (!LISTED && EPI == kEpiMinDist) {                     // (not listed: a single pass)
    for (int off = 32; off > 0; off >>= 1) run_min = fminf(run_min, __shfl_xor(run_min, off, 64));
    if (lane == 0) atomicMin(a.best, (unsigned long long)__float_as_uint(fmaxf(run_min, 0.f)));   // non-negative floats order like their bits
  }
  }   // segments of the row's tile list
  if (!LISTED) break;
  }   // rows
}

// ---------------------------------------------------------------------------------------------
// Relation-factorised dense L2 join (optional mode).  For the TransE distance of Section 4.3,
//     ||h + r - t||^2 = ||h - t||^2 + 2 r.h - 2 r.t + ||r||^2,
// and the only part that needs a d-long contraction per (h, t) pair, ||h - t||^2, does not depend on the
// relation (the observation Section 5.2 makes for the tail side, taken one step further).  One block keeps
// a 256-row head tile in LDS, forms the 256 x 256 tile G = ||h~ - t~||^2 ONCE with the matrix pipes (plain
// entity rows on both sides, same augmented-K operands as the other forms), and then walks the relations of
// the batch with vector arithmetic only: per relation and element one addition (G + 2 r.h) and half a
// three-way minimum, the result compared against lim_r + 2 r.t per tail column.  The products r.e are a
// float32 matrix u[r][slot] made beforehand by a tiled kernel.  Elements that pass go to the same exact
// double-precision re-scoring as everywhere else, so the result set is unchanged.
// Filter threshold: see k_fact_params.  LDS: the head tile (KS * 16 KiB) and 2 r.h of `rc` relations at a
// time (rc KiB).
struct JoinFactArgs {
  const uint16_t* A;         // staged head operands of the plain entity rows: [KS][Nslots][32]
  const uint16_t* B;         // staged tail operands: [KS][Nslots][32]
  const float* u;            // [RB][Nslots] r . e (float32, from the caller's rows)
  const float* limr;         // [RB] threshold on G + 2 r.h - 2 r.t, i.e. thr_r - ||r||^2
  int64_t Nslots;
  int KS, k16;
  int nH, nT;
  int r0, RB;
  int rc;                    // relations per LDS chunk
  RecheckCtx cx;
};

template <int WGM, int WGN>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void k_join_l2_fact(const JoinFactArgs a) {
  constexpr int BM = 256, BN = 256;
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int LA = (BM * 4) / NT;
  constexpr int ASZ = BM * kSliceK;
  constexpr int ROWB = kSliceK * 2;
  static_assert(LA * NT == BM * 4, "tile rows must divide over the threads");

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // [KS][BM][32] head slices, then float uh[rc][BM]
  const int KS = a.KS;
  float* uh = (float*)(lds + (size_t)KS * ASZ);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  const int tH = (int)blockIdx.x;
  const int t_begin = (int)(((int64_t)a.nT * blockIdx.y) / gridDim.y);
  const int t_end = (int)(((int64_t)a.nT * (blockIdx.y + 1)) / gridDim.y);
  if (t_end <= t_begin) return;
  const int64_t slice_bytes = a.Nslots * ROWB;

  // ---- head tile: all K slices into LDS, once ----
  {
    const char* Abase = (const char*)a.A + (int64_t)tH * BM * ROWB;
    const uint32_t voff = (uint32_t)tid * 16u;
    const int st0 = (tid >> 2) * kSliceK + (((tid & 3) ^ lds_swizzle(tid >> 2)) * 8);
    constexpr int st_step = (NT / 4) * kSliceK;
    for (int ks = 0; ks < KS; ++ks) {
      uint4 t[LA];
#pragma unroll
      for (int i = 0; i < LA; ++i) t[i] = *(const uint4*)(Abase + (int64_t)ks * slice_bytes + voff + (uint32_t)(i * NT * 16));
#pragma unroll
      for (int i = 0; i < LA; ++i) *(uint4*)(&lds[ks * ASZ + st0 + i * st_step]) = t[i];
    }
  }
  __syncthreads();

  const int rsw = lds_swizzle(lane & 31);
  const int rd_a = (wm * WTM + (lane & 31)) * kSliceK + (((lane >> 5) ^ rsw) * 8);
  const int rd_step = (((lane >> 5) ^ rsw) & 2) ? -16 : 16;
  const uint32_t boff = (uint32_t)((wn * WTN + (lane & 31)) * ROWB + (lane >> 5) * 16);
  const int last_two = (a.k16 - (KS - 1) * 2) >= 2;
  // this lane's rows inside a 32-row block: 8 * (v / 4) + 4 * (lane / 32) + (v % 4); its column: lane % 32
  const int urow = wm * WTM + 4 * (lane >> 5);

  for (int tT = t_begin; tT < t_end; ++tT) {
    // ---- G = ||h~ - t~||^2 for the 256 x 256 tile: tail fragments straight from the staged array ----
    f32x16_t acc[TM][TN];
    const char* pB = (const char*)a.B + (int64_t)tT * BN * ROWB + boff;
    for (int ks = 0; ks < KS; ++ks) {
      const uint16_t* Ac = lds + ks * ASZ + rd_a;
      const bool two = ks < KS - 1 || last_two;
      bf16x8_t fb0[TN], fb1[TN], fa[TM];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        fb0[j] = *(const bf16x8_t*)(pB + j * 32 * ROWB);
        fb1[j] = *(const bf16x8_t*)(pB + j * 32 * ROWB + 32);
      }
      pB += slice_bytes;
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK);
      if (ks == 0) {
        const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb0[j], zero16, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb0[j], acc[i][j], 0, 0, 0);
      }
      if (two) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8_t*)(Ac + i * 32 * kSliceK + rd_step);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb1[j], acc[i][j], 0, 0, 0);
      }
    }

    // ---- the relations of the batch, rc at a time: 2 r.h of the head rows through LDS ----
    const int64_t tcol0 = (int64_t)tT * BN + wn * WTN + (lane & 31);     // this lane's column of block j: + 32 j
    for (int rl0 = 0; rl0 < a.RB; rl0 += a.rc) {
      const int nr = a.RB - rl0 < a.rc ? a.RB - rl0 : a.rc;
      __syncthreads();                                                    // the previous chunk has been read
      for (int e = tid; e < nr * BM; e += NT) {
        const int q = e / BM, row = e - q * BM;
        uh[q * BM + row] = 2.f * a.u[(int64_t)(rl0 + q) * a.Nslots + (int64_t)tH * BM + row];
      }
      __syncthreads();
      // the per-column part of the threshold (lim_r + 2 r.t) is fetched one relation ahead of its use
      float nlimr = a.limr[rl0], nut[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) nut[j] = a.u[(int64_t)rl0 * a.Nslots + tcol0 + 32 * j];
      for (int q = 0; q < nr; ++q) {
        const int rl = rl0 + q;
        float lim[TN], mn[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          lim[j] = nlimr + 2.f * nut[j];
          mn[j] = 3e38f;
        }
        {
          const int rn = q + 1 < nr ? rl + 1 : rl;              // the last one re-reads itself
          nlimr = a.limr[rn];
#pragma unroll
          for (int j = 0; j < TN; ++j) nut[j] = a.u[(int64_t)rn * a.Nslots + tcol0 + 32 * j];
        }
        const float* uq = uh + q * BM + urow;
        // per element one addition and half a three-way minimum; the 2 r.h values of this lane's rows come
        // from LDS, four rows per read (two addresses per wave), two reads ahead of their use
        constexpr int NH4 = TM * 4;
        float4 hq0 = *(const float4*)(uq), hq1 = *(const float4*)(uq + 8);
#pragma unroll
        for (int k = 0; k < NH4; ++k) {
          const int i = k >> 2, vg = k & 3;                          // rows v = 4 vg .. 4 vg + 3 of block i
          const float4 hh = hq0;
          hq0 = hq1;
          if (k + 2 < NH4) hq1 = *(const float4*)(uq + ((k + 2) >> 2) * 32 + 8 * ((k + 2) & 3));
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            mn[j] = fminf(fminf(mn[j], acc[i][j][4 * vg + 0] + hh.x), acc[i][j][4 * vg + 1] + hh.y);
            mn[j] = fminf(fminf(mn[j], acc[i][j][4 * vg + 2] + hh.z), acc[i][j][4 * vg + 3] + hh.w);
          }
        }
        bool any = false;
#pragma unroll
        for (int j = 0; j < TN; ++j) any |= mn[j] <= lim[j];
        if (__builtin_amdgcn_ballot_w64(any) == 0ull) continue;
        // rare: the elements of this relation that pass, then the exact path.  MFMA 32x32 accumulator layout:
        // register v of lane l holds row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
        const int64_t hbase = (int64_t)tH * BM + wm * WTM;
        const int64_t tbase = (int64_t)tT * BN + wn * WTN;
        constexpr int NW = (TM * TN + 3) / 4;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          unsigned long long cm = 0ull;
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            const int tile = w * 4 + qq;
            if (tile < TM * TN) {
              const int i = tile / TN, j = tile % TN;
#pragma unroll
              for (int v = 0; v < 16; ++v)
                if (acc[i][j][v] + uq[i * 32 + 8 * (v >> 2) + (v & 3)] <= lim[j]) cm |= 1ull << (qq * 16 + v);
            }
          }
          if (__builtin_amdgcn_ballot_w64(cm != 0ull) == 0ull) continue;
          recheck_and_emit(cm, a.r0 + rl, a.cx, [=](int e, int src, int64_t& hslot, int64_t& tslot) {
            const int tile = w * 4 + (e >> 4), v = e & 15;
            const int i = tile / TN, j = tile % TN;
            hslot = hbase + i * 32 + 8 * (v >> 2) + 4 * (src >> 5) + (v & 3);
            tslot = tbase + j * 32 + (src & 31);
          });
        }
      }
    }
  }
}

// Per-relation filter thresholds of the factorised join: limr[rl] = thr_r - ||r||^2, where a true hit has
//     G + 2 r.h - 2 r.t + ||r||^2 <= thr_r = delta^2 + m (2 (delta + ||r||) + m) + e_acc + e_u:
// G is taken on bf16-rounded rows, which moves ||h - t|| by at most m = 2^-8 1.01 (max||h~|| + max||t~||)
// (m = 0 for bf16 storage, where rounding changes nothing), and ||h - t|| <= delta + ||r|| for a hit, hence the
// first term; e_acc bounds the float32 accumulation of G as in k_join_params; e_u bounds the float32 error of
// the two products (d + 8) 2^-24 ||r|| ||e|| each, doubled, and of the final sums.
__global__ __launch_bounds__(256) void k_fact_params(const DevCounters* cnt, const float* __restrict__ rn, int RB, float delta,
                                                     int dtype, int d, int kp, float* __restrict__ limr) {
  __shared__ float sm[2];
  if (threadIdx.x < 64) {
    float ma = 0.f, mb = 0.f;
    for (int i = threadIdx.x; i < 1024; i += 64) {
      ma = fmaxf(ma, __uint_as_float(cnt->max_a[i]));
      mb = fmaxf(mb, __uint_as_float(cnt->max_b[i]));
    }
    for (int off = 32; off > 0; off >>= 1) {
      ma = fmaxf(ma, __shfl_xor(ma, off, 64));
      mb = fmaxf(mb, __shfl_xor(mb, off, 64));
    }
    if (threadIdx.x == 0) { sm[0] = ma; sm[1] = mb; }
  }
  __syncthreads();
  const float ma = sm[0], mb = sm[1];
  const int rl = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (rl >= RB) return;
  if (delta < 0.f) { limr[rl] = -3e38f; return; }
  const float na = sqrtf(ma) * 1.01f, nb = sqrtf(mb) * 1.01f;
  const float m = dtype == KGC_BF16 ? 0.f : (1.01f / 256.f) * (na + nb);
  const float rnorm = sqrtf(rn[rl]) * 1.0001f;
  const float eacc = (float)(kp + 16) * 1.2e-7f * 2.f * (ma + mb);
  const float eu = 4.f * (float)(d + 12) * 6e-8f * rnorm * (na + nb) + 1e-6f * (rn[rl] + ma + mb);
  const float thr = (delta * delta + m * (2.f * (delta + rnorm) + m) + eacc + eu) * (1.f + 1e-6f);
  limr[rl] = thr - rn[rl];
}

// ---------------------------------------------------------------------------------------------
// Top-1 search (the smallest triple distance, Section 3.3).  Three small kernels around the join:
//   k_top1_sample  exact distances of `n` pseudo-random triples (one per 16-lane group), minimum by atomicMin
//                  on the bits of the non-negative double: an upper bound of the top-1 distance to start from;
//   k_top1_min     over the records a join returned: pass 0 the minimum of (distance bits << 32 | r), pass 1,
//                  among the records that attain it, the minimum of (h << 32 | t);
//   k_top1_exact   the double-precision distance of the chosen triple.
struct Top1State {
  unsigned long long sample_min;   // bits of a double
  unsigned long long key_dr;       // (float distance bits << 32) | r
  unsigned long long key_ht;       // (h << 32) | t
  double dist;                     // exact distance of (key_ht, r of key_dr)
  unsigned long long sub_min;      // float bits of the smallest squared distance the sub-sampled dense pass saw
  double sub_bound;                // the distance bound that follows from it
};

__device__ __forceinline__ uint32_t top1_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

__global__ __launch_bounds__(256) void k_top1_sample(RecheckCtx cx, int64_t N, int r_begin, int R, int n, int no_self,
                                                     Top1State* st, double* all = nullptr) {
  const int64_t g = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4;
  const int sub = threadIdx.x & 15;
  if (g >= n) return;                                   // whole 16-lane groups leave together
  const uint32_t a = top1_hash((uint32_t)g * 3u + 1u), b = top1_hash((uint32_t)g * 3u + 2u), c = top1_hash((uint32_t)g * 3u + 3u);
  const int32_t h = (int32_t)(((uint64_t)a * (uint64_t)N) >> 32);
  int32_t t = (int32_t)(((uint64_t)b * (uint64_t)N) >> 32);
  const int32_t r = r_begin + (int32_t)(((uint64_t)c * (uint64_t)R) >> 32);      // R relations from r_begin on
  if (no_self && t == h) t = (t + 1 == N) ? 0 : t + 1;  // N >= 2 is checked on the host
  const double dist = group16_exact_dist(cx, h, r, t, sub);
  if (sub == 0) {
    atomicMin(&st->sample_min, (unsigned long long)__double_as_longlong(dist));
    if (all) all[g] = dist;                               // top-k: the whole sample goes to the host
  }
}

__global__ __launch_bounds__(256) void k_top1_min(const kgc_triple* __restrict__ rec, const unsigned long long* __restrict__ count,
                                                  unsigned long long cap, int pass, Top1State* st) {
  const unsigned long long n = *count < cap ? *count : cap;
  unsigned long long best = ~0ull;
  const unsigned long long want = st->key_dr;           // pass 1: written by pass 0, an earlier launch
  for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (unsigned long long)gridDim.x * blockDim.x) {
    const kgc_triple x = rec[i];
    const unsigned long long kdr = ((unsigned long long)__float_as_uint(x.dist) << 32) | (uint32_t)x.r;
    if (pass == 0) best = kdr < best ? kdr : best;
    else if (kdr == want) {
      const unsigned long long kht = ((unsigned long long)(uint32_t)x.h << 32) | (uint32_t)x.t;
      best = kht < best ? kht : best;
    }
  }
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)(best & 0xffffffffull), off, 64);
    const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(best >> 32), off, 64);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    best = o < best ? o : best;
  }
  if ((threadIdx.x & 63) == 0 && best != ~0ull) atomicMin(pass == 0 ? &st->key_dr : &st->key_ht, best);
}

// Disjoint head and tail samples for the sub-sampled dense pass: 2 m entities evenly spread over [0, N),
// even positions to the heads, odd positions to the tails (so the pass scores no self pair); N >= 2 m.
__global__ void k_top1_pick(int64_t N, int m, int32_t* heads, int32_t* tails) {
  const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= m) return;
  heads[i] = (int32_t)(((int64_t)(2 * i) * N) / (2 * (int64_t)m));
  tails[i] = (int32_t)(((int64_t)(2 * i + 1) * N) / (2 * (int64_t)m));
}

// The smallest squared distance of the sub-sampled pass is taken on bf16-rounded rows with float32
// accumulation; the true distance of that pair is at most sqrt(D + e_acc) + m (same m and e_acc as the join's
// filter threshold, see k_join_params), which bounds the top-1 distance from above.
__global__ __launch_bounds__(64) void k_top1_bound(const DevCounters* cnt, int dtype, int kp, Top1State* st) {
  float ma = 0.f, mb = 0.f;
  for (int i = threadIdx.x; i < 1024; i += 64) {
    ma = fmaxf(ma, __uint_as_float(cnt->max_a[i]));
    mb = fmaxf(mb, __uint_as_float(cnt->max_b[i]));
  }
  for (int off = 32; off > 0; off >>= 1) {
    ma = fmaxf(ma, __shfl_xor(ma, off, 64));
    mb = fmaxf(mb, __shfl_xor(mb, off, 64));
  }
  if (threadIdx.x != 0) return;
  const float D = __uint_as_float((uint32_t)st->sub_min);
  const float u = 1.01f / 256.f;
  const float m = u * (sqrtf(ma) * 1.01f + (dtype == KGC_BF16 ? 0.f : sqrtf(mb) * 1.01f));
  const float eacc = (float)(kp + 16) * 1.2e-7f * 2.f * (ma + mb);
  st->sub_bound = ((double)sqrtf(D + eacc) + (double)m) * (1.0 + 1e-5);
}

// ---- top-k: the k smallest of the n records a join returned, by radix select on the float bits of the
// distance (non-negative floats order like their bits), 8 bits per pass from the top.  State on the device:
//   prefix / mask  the bits fixed so far;  need  how many records are still wanted among those that match.
struct TopkState {
  unsigned int hist[256];
  unsigned int prefix, mask;
  unsigned long long need;        // records still to take among the keys that match the prefix
  unsigned long long taken_less;  // emit: records with a smaller key written so far
  unsigned long long taken_eq;    // emit: records with the k-th key written so far
};

__global__ void k_topk_init(TopkState* ts, unsigned long long k) {
  const int i = threadIdx.x;
  if (i < 256) ts->hist[i] = 0u;
  if (i == 0) { ts->prefix = 0u; ts->mask = 0u; ts->need = k; ts->taken_less = 0ull; ts->taken_eq = 0ull; }
}

__global__ __launch_bounds__(256) void k_topk_hist(const kgc_triple* __restrict__ rec, const unsigned long long* __restrict__ count,
                                                   unsigned long long cap, int shift, TopkState* ts) {
  __shared__ unsigned int h[256];
  h[threadIdx.x] = 0u;
  __syncthreads();
  const unsigned long long n = *count < cap ? *count : cap;
  const unsigned int prefix = ts->prefix, mask = ts->mask;
  for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (unsigned long long)gridDim.x * blockDim.x) {
    const unsigned int key = __float_as_uint(rec[i].dist);
    if ((key & mask) == prefix) atomicAdd(&h[(key >> shift) & 255u], 1u);
  }
  __syncthreads();
  if (h[threadIdx.x]) atomicAdd(&ts->hist[threadIdx.x], h[threadIdx.x]);
}

// one thread: which digit holds the need-th record among the matching keys; fix it and clear the histogram
__global__ void k_topk_digit(int shift, TopkState* ts) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  unsigned long long need = ts->need, acc = 0ull;
  int dsel = 255;
  for (int b = 0; b < 256; ++b) {
    const unsigned long long c = ts->hist[b];
    if (acc + c >= need) { dsel = b; break; }
    acc += c;
  }
  ts->need = need - acc;            // still wanted inside the chosen digit
  ts->prefix |= (unsigned int)dsel << shift;
  ts->mask |= 255u << shift;
  for (int b = 0; b < 256; ++b) ts->hist[b] = 0u;
}

// after four passes prefix is the k-th smallest key T and need the number of records with key == T to take:
// every record below T goes out, and the first `need` of those at T that get there
__global__ __launch_bounds__(256) void k_topk_emit(const kgc_triple* __restrict__ rec, const unsigned long long* __restrict__ count,
                                                   unsigned long long cap, unsigned long long k, TopkState* ts,
                                                   kgc_triple* __restrict__ out) {
  const unsigned long long n = *count < cap ? *count : cap;
  const unsigned int T = ts->prefix;
  const unsigned long long need_eq = ts->need;
  const unsigned long long n_less = (n < k ? n : k) - (need_eq < (n < k ? n : k) ? need_eq : (n < k ? n : k));
  for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (unsigned long long)gridDim.x * blockDim.x) {
    const kgc_triple x = rec[i];
    const unsigned int key = __float_as_uint(x.dist);
    if (n <= k) { out[i] = x; continue; }                 // fewer records than asked for: all of them
    if (key < T) out[atomicAdd(&ts->taken_less, 1ull)] = x;
    else if (key == T) {
      const unsigned long long j = atomicAdd(&ts->taken_eq, 1ull);
      if (j < need_eq) out[n_less + j] = x;
    }
  }
}

__global__ __launch_bounds__(64) void k_top1_exact(RecheckCtx cx, Top1State* st) {
  const int sub = threadIdx.x & 15;
  const int32_t r = (int32_t)(uint32_t)(st->key_dr & 0xffffffffull);
  const int32_t h = (int32_t)(uint32_t)(st->key_ht >> 32), t = (int32_t)(uint32_t)(st->key_ht & 0xffffffffull);
  const double dist = group16_exact_dist(cx, h, r, t, sub);
  if (threadIdx.x == 0) st->dist = dist;
}

// ---------------------------------------------------------------------------------------------
struct JoinL1Args {
  const JoinParams* prm;
  int64_t Nslots;
  int nH, nT;
  int r0, RB;
  const uint32_t* row_start;   // NULL: dense (one block per tile, grid = (nT, nH, RB)); else see JoinStreamArgs
  const uint32_t* row_count;
  const uint32_t* cols;
  const uint32_t* active_rows;
  const unsigned int* n_active;
  RecheckCtx cx;
};

// Kernel 3.  One block of 256 threads scores 128 x 128 tiles of (heads, tails) for one relation in
// float32 vector arithmetic only: acc += |(h_k + r_k) - t_k| (Section 4.3's dist for p = 1).  A tile is
// staged through LDS in 16-dimension slices, dimension-major, a = h + r formed while staging; each
// thread keeps an 8 x 8 block of sums in registers (two 4-row groups x two 4-column groups).  In pruned
// mode the block walks the surviving tail tiles of its (relation, head tile) row.
constexpr int kL1Tile = 128;
constexpr int kL1K = 16;
__global__ __launch_bounds__(256, 3) void k_join_l1(const JoinL1Args a) {
  constexpr int BM = kL1Tile, BN = kL1Tile, BK = kL1K;
  __shared__ __attribute__((aligned(16))) float As[BK][BM];
  __shared__ __attribute__((aligned(16))) float Bs[BK][BN];
  __shared__ int32_t hent[BM], tent[BN];
  __shared__ BlockQueue queue;

  const int tid = threadIdx.x, wave = tid >> 6;
  if (tid == 0) { queue.count = 0u; queue.pending = 0u; queue.flag = 0u; queue.nhits = 0u; }   // published by the first barrier
  for (unsigned int row_i = blockIdx.x;; row_i += gridDim.x) {
  int tH, rl, t_begin, t_end;
  const uint32_t* cols = nullptr;
  if (a.row_start) {
    if (row_i >= *a.n_active) break;
    const int64_t row = (int64_t)a.active_rows[row_i];
    rl = (int)(row / a.nH); tH = (int)(row - (int64_t)rl * a.nH);
    t_begin = (int)a.row_start[row]; t_end = t_begin + (int)a.row_count[row];
    cols = a.cols;
    __syncthreads();                      // the previous row is done with hent
  } else {
    t_begin = (int)blockIdx.x; t_end = t_begin + 1; tH = (int)blockIdx.y; rl = (int)blockIdx.z;
  }
  if (t_end <= t_begin) break;
  const int r = a.r0 + rl;
  const int d = a.cx.d, dtype = a.cx.dtype;
  const float thr = a.prm->thr;
  const int tx = tid & 15, ty = tid >> 4;
  // staging assignment: thread -> (row = tid / 2, eight dimensions starting at (tid % 2) * 8)
  const int srow = tid >> 1, sk0 = (tid & 1) * 8;
  const int64_t ro = (int64_t)r * a.cx.rstride;
  if (tid < BM) hent[tid] = a.cx.slot_ent[(int64_t)tH * BM + tid];

#pragma unroll 1
  for (int ti = t_begin; ti < t_end; ++ti) {
    const int tT = cols ? (int)cols[ti] : ti;
    __syncthreads();                        // previous tile done with tent / As / Bs
    if (tid >= BM) tent[tid - BM] = a.cx.slot_ent_t[(int64_t)tT * BN + (tid - BM)];
    __syncthreads();
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    const int he = hent[srow], te = tent[srow];
    const int64_t ho = (int64_t)r * a.cx.hstride + (int64_t)(he < 0 ? 0 : he) * d,
                  to = (int64_t)r * a.cx.tstride + (int64_t)(te < 0 ? 0 : te) * d;

#pragma unroll 1
    for (int k0 = 0; k0 < d; k0 += BK) {
      float va[8], vb[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int k = k0 + sk0 + q;
        const bool in = k < d;
        va[q] = in ? ld_elem(a.cx.E, ho + k, dtype) + ld_elem(a.cx.Rv, ro + k, dtype) : 0.f;
        vb[q] = in ? ld_elem(a.cx.Et, to + k, dtype) : 0.f;
      }
      __syncthreads();                      // previous slice fully consumed
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        As[sk0 + q][srow] = va[q];
        Bs[sk0 + q][srow] = vb[q];
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < BK; ++k) {
        const float4 a0 = *(const float4*)(&As[k][ty * 4]);
        const float4 a1 = *(const float4*)(&As[k][64 + ty * 4]);
        const float4 b0 = *(const float4*)(&Bs[k][tx * 4]);
        const float4 b1 = *(const float4*)(&Bs[k][64 + tx * 4]);
        const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        const float bv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[i][j] += fabsf(av[i] - bv[j]);
      }
    }

    unsigned long long cm[1] = {0ull};
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (acc[i][j] <= thr) cm[0] |= 1ull << (i * 8 + j);
    // the exact path is entered by the whole block or not at all
    if (__builtin_amdgcn_ballot_w64(cm[0] != 0ull) != 0ull && (tid & 63) == 0) queue.flag = 1u;
    __syncthreads();
    if (queue.flag) {
      const int64_t hbase = (int64_t)tH * BM, tbase = (int64_t)tT * BN;
      block_recheck<4, 1, 1>(cm, r, a.cx, &queue, [=](int e, int src, int64_t& hslot, int64_t& tslot) {
        const int stid = wave * 64 + src;
        const int sx = stid & 15, sy = stid >> 4;
        const int i = e >> 3, j = e & 7;
        hslot = hbase + (i >> 2) * 64 + sy * 4 + (i & 3);
        tslot = tbase + (j >> 2) * 64 + sx * 4 + (j & 3);
      });
    }
  }
  if (!a.row_start) break;
  }   // rows
}

}  // namespace kgc

// Block-level pruning for the TransE completion join (gfx950).
//
// The paper filters pairs with one pivot p: dist(a, b) >= |dist(p, a) - dist(p, b)| (Lemma 1, Section 4.4)
// and turns that into index ranges over pivot-sorted lists (Lemma 2).  On embeddings whose norms
// concentrate, the single zero pivot of Section 4.5 separates little, so this build applies the same
// triangle-inequality argument with LOCAL pivots: entities are grouped around pivot entities, stored
// group by group, and every 32-row micro-tile m gets a centre c_m and a radius rho_m >= dist(e, c_m)
// for its rows.  For a = h + r with h in micro-tile H and b = t in micro-tile T,
//     dist(a, b) >= dist(c_H + r, c_T) - rho_H - rho_T          (triangle inequality, twice)
// so the pair of micro-tiles is skipped when that bound exceeds delta.  A join tile is evaluated iff one
// of its micro-tile pairs survives.  All of it is done in the metric of the join (L1 or L2); bounds are
// computed in float32 and widened by a relative slack so that rounding can only keep more, never drop.
#pragma once
#include "kgc_device.h"

namespace kgc {

constexpr int kMicro = 32;                 // rows per micro-tile (the MFMA tile height)
constexpr int kGroupRounds = 6;            // covering rounds
constexpr int kPivotsPerRound = 4096;      // pivots drawn from the uncovered entities per round
constexpr int kMaxGroups = kGroupRounds * kPivotsPerRound;
constexpr int kSmallGroup = 16;            // smaller groups are packed, unpadded, into the tail region
constexpr float kBoundSlack = 2e-4f;       // relative widening of float32 distance sums (d <= 960 terms)

struct GroupState {
  int32_t n_unc;        // uncovered entities in the current list
  int32_t n_unc_next[2]; // ... appended to the next list, by the round's parity (a round's start reads the count the
                        // round before left and clears its own)
  int32_t n_piv;        // pivots of the current round
  int32_t n_groups;     // groups formed so far
  int32_t n_slots;      // rows after layout, multiple of the slot alignment
  int32_t tail_base;    // first slot of the unpadded tail region
  int32_t tail_fill;    // running count of rows placed in the tail region
  int32_t n_big;        // groups of at least kSmallGroup rows: each is one unit of the two-level bound test
};

// Start of a round: pivots are an even-stride sample (one in 2^shift, at most kPivotsPerRound) of the
// uncovered list; nearest-pivot records are reset.
// `best` is indexed by the position in the uncovered list, or (by_entity) by the entity itself; the pivot
// list is padded with -1 up to kPivotsPerRound (the grid covers max(N, kPivotsPerRound) threads).
// The first round (init_N > 0) also sets up the state: every entity uncovered and in no group.  A later round first
// closes the one before it (its pivots become groups, the entities it left uncovered are this round's list): what
// the threads read of the state is not what thread 0 writes.
__global__ void k_round_begin(GroupState* gs, int32_t* unc, int32_t* piv_ent, unsigned long long* best,
                              int shift, int by_entity, int64_t init_N, int32_t* group_of, int round) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool first = init_N > 0;
  const int n_unc = first ? (int)init_N : gs->n_unc_next[(round & 1) ^ 1];
  int n_piv = n_unc >> shift;
  n_piv = n_piv < 1 ? (n_unc > 0 ? 1 : 0) : n_piv;
  n_piv = n_piv < kPivotsPerRound ? n_piv : kPivotsPerRound;
  if (first && i < n_unc) { unc[i] = (int32_t)i; group_of[i] = -1; }
  if (i < kPivotsPerRound) {
    const int64_t pos = i < n_piv ? (int64_t)i * n_unc / n_piv : -1;   // n_piv > 0 where read
    piv_ent[i] = pos < 0 ? -1 : (first ? (int32_t)pos : unc[pos]);
  }
  if (i < n_unc) best[by_entity ? (first ? (int32_t)i : unc[i]) : i] = ~0ull;
  if (i == 0) {
    if (first) { gs->n_groups = 0; gs->n_slots = 0; gs->tail_base = 0; gs->tail_fill = 0; gs->n_big = 0; }
    else gs->n_groups += gs->n_piv;                        // the round before
    gs->n_unc = n_unc; gs->n_piv = n_piv; gs->n_unc_next[round & 1] = 0;
  }
}

// End of a round: an uncovered entity joins the group of the pivot the assignment found within tau, if any.
__global__ void k_round_commit(GroupState* gs, const int32_t* unc, const unsigned long long* best,
                               int32_t* group_of, int32_t* unc_next, int by_entity, int round) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= gs->n_unc) return;
  const int ent = unc[i];
  const unsigned long long b = best[by_entity ? ent : i];
  if (b != ~0ull) group_of[ent] = gs->n_groups + (int)(uint32_t)(b >> 32);
  else unc_next[atomicAdd(&gs->n_unc_next[round & 1], 1)] = ent;
}

// before the layout: group sizes and fill counts to zero, every slot to "padding"; the last round (number last_round)
// is closed
__global__ void k_group_clear(int32_t* gsize, int32_t* gfill, int n_groups_max, int32_t* slot_ent, int64_t n_slots,
                              GroupState* gs, int last_round) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) {
    gs->n_groups += gs->n_piv;
    gs->n_unc = gs->n_unc_next[last_round & 1];
    gs->n_piv = 0;
  }
  if (i < n_groups_max) { gsize[i] = 0; gfill[i] = 0; }
  if (i < n_slots) slot_ent[i] = -1;
}

__global__ void k_group_hist(const int32_t* group_of, int64_t N, int32_t* gsize) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N && group_of[i] >= 0) atomicAdd(&gsize[group_of[i]], 1);
}

// Slot layout: groups of at least kSmallGroup rows start on a micro-tile boundary and are padded to one;
// all other rows follow, packed.  One block of 1024 threads: each thread owns a contiguous run of groups,
// an exclusive scan over the threads' padded sizes gives the run offsets.
// The padded groups are also numbered 0 .. n_big - 1 in slot order and their micro-tile ranges written to
// unit_first / unit_n: they are the units of the two-level bound test.
__global__ __launch_bounds__(1024) void k_group_layout(GroupState* gs, const int32_t* gsize, int32_t* goff, int64_t N,
                                                       int slot_align, int32_t* unit_first, int32_t* unit_n) {
  __shared__ int part[1024];
  __shared__ int placed_part[1024];
  __shared__ int big_part[1024];
  const int tid = threadIdx.x;
  const int G = gs->n_groups;
  const int per = (G + 1023) / 1024;
  const int g0 = tid * per, g1 = (g0 + per < G) ? g0 + per : G;
  int sum = 0, placed = 0, nbig = 0;
  for (int g = g0; g < g1; ++g) {
    const int sz = gsize[g];
    if (sz >= kSmallGroup) { sum += (sz + kMicro - 1) / kMicro * kMicro; placed += sz; ++nbig; }
  }
  part[tid] = sum;
  placed_part[tid] = placed;
  big_part[tid] = nbig;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {          // inclusive scan, Hillis-Steele
    const int v = tid >= off ? part[tid - off] : 0;
    const int w = tid >= off ? placed_part[tid - off] : 0;
    const int x = tid >= off ? big_part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    placed_part[tid] += w;
    big_part[tid] += x;
    __syncthreads();
  }
  int cur = part[tid] - sum;                           // exclusive prefix of this thread's run
  int ui = big_part[tid] - nbig;
  for (int g = g0; g < g1; ++g) {
    const int sz = gsize[g];
    if (sz >= kSmallGroup) {
      const int padded = (sz + kMicro - 1) / kMicro * kMicro;
      goff[g] = cur;
      unit_first[ui] = cur / kMicro;
      unit_n[ui] = padded / kMicro;
      ++ui;
      cur += padded;
    } else {
      goff[g] = -1;
    }
  }
  if (tid == 1023) {
    const int total_padded = part[1023];
    gs->n_big = big_part[1023];
    gs->tail_base = total_padded;
    gs->tail_fill = 0;
    const int64_t total = (int64_t)total_padded + (N - placed_part[1023]);
    gs->n_slots = (int32_t)((total + slot_align - 1) / slot_align * slot_align);
  }
}

__global__ void k_scatter_slots(GroupState* gs, const int32_t* group_of, const int32_t* goff, int32_t* gfill,
                                int64_t N, int32_t* slot_ent) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  const int g = group_of[i];
  int slot;
  if (g >= 0 && goff[g] >= 0) slot = goff[g] + atomicAdd(&gfill[g], 1);
  else slot = gs->tail_base + atomicAdd(&gs->tail_fill, 1);
  slot_ent[slot] = (int32_t)i;
}

// One wave per micro-tile: centre = mean of its rows, radius = max distance of a row to the centre (in
// the join's metric), widened for float32 rounding.  An empty micro-tile gets radius -1.
// The rows are read once, 64 dimensions at a time with the lanes on consecutive dimensions: the 32 loads of a chunk
// are independent of each other (one memory round trip), the chunk's centre values come from their sum, and each
// row's distance to the centre grows by its part of the chunk; the 32 row sums are then added across the lanes by a
// halving exchange (32 shuffles).
template <int P>
__global__ __launch_bounds__(64) void k_micro_summary(const void* __restrict__ E, int dtype, int d,
                                                      const int32_t* __restrict__ slot_ent, int64_t n_micro,
                                                      float* __restrict__ cent, float* __restrict__ rad,
                                                      float* __restrict__ cnorm, int r0 = 0, int64_t rel_stride = 0) {
  // blockIdx.y: relation of a batch, for per-relation rows E[(r0 + y) * rel_stride + ...] (summaries then lie
  // relation after relation); one relation and rel_stride 0 for the TransE join
  static_assert(kMicro == 32, "the row sums below are laid out for 32 rows");
  const int64_t m = blockIdx.x;
  if (m >= n_micro) return;
  const int lane = threadIdx.x;
  E = (const char*)E + (int64_t)(r0 + (int)blockIdx.y) * rel_stride * (dtype == KGC_BF16 ? 2 : 4);
  cent += (int64_t)blockIdx.y * n_micro * d; rad += (int64_t)blockIdx.y * n_micro; cnorm += (int64_t)blockIdx.y * n_micro;
  const int32_t ent_l = lane < kMicro ? slot_ent[m * kMicro + lane] : -1;
  const int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(ent_l >= 0));
  float* c = cent + m * d;
  if (cnt == 0) {
    for (int k = lane; k < d; k += 64) c[k] = 0.f;
    if (lane == 0) { rad[m] = -1.f; cnorm[m] = 0.f; }
    return;
  }
  const float inv = 1.f / (float)cnt;
  float c2 = 0.f;
  float rs[kMicro];                                   // this lane's part of every row's distance to the centre
#pragma unroll
  for (int q = 0; q < kMicro; ++q) rs[q] = 0.f;
  for (int k0 = 0; k0 < d; k0 += 64) {
    const int k = k0 + lane;
    float v[kMicro];
#pragma unroll
    for (int q = 0; q < kMicro; ++q) v[q] = 0.f;
    if (k < d) {
#pragma unroll
      for (int q = 0; q < kMicro; ++q) {
        const int32_t ent = __builtin_amdgcn_readlane(ent_l, q);
        if (ent >= 0) v[q] = ld_elem(E, (int64_t)ent * d + k, dtype);
      }
      float sum = 0.f;
#pragma unroll
      for (int q = 0; q < kMicro; ++q) sum += v[q];
      const float ck = sum * inv;
      c[k] = ck;
      c2 += ck * ck;
#pragma unroll
      for (int q = 0; q < kMicro; ++q) {
        const float x = v[q] - ck;
        if (__builtin_amdgcn_readlane(ent_l, q) >= 0) rs[q] += (P == 2) ? x * x : fabsf(x);
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) c2 += __shfl_xor(c2, off, 64);
  if (lane == 0) cnorm[m] = sqrtf(c2) * (1.f + kBoundSlack);
  // row totals: after the five halving steps lane l holds the sum of row 16 b5 + 8 b4 + 4 b3 + 2 b2 + b1 (bits of l)
  float a16[16], a8[8], a4[4], a2[2], a1;
  {
    const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
#pragma unroll
    for (int i = 0; i < 16; ++i) a16[i] = (b5 ? rs[i + 16] : rs[i]) + __shfl_xor(b5 ? rs[i] : rs[i + 16], 32, 64);
#pragma unroll
    for (int i = 0; i < 8; ++i) a8[i] = (b4 ? a16[i + 8] : a16[i]) + __shfl_xor(b4 ? a16[i] : a16[i + 8], 16, 64);
#pragma unroll
    for (int i = 0; i < 4; ++i) a4[i] = (b3 ? a8[i + 4] : a8[i]) + __shfl_xor(b3 ? a8[i] : a8[i + 4], 8, 64);
#pragma unroll
    for (int i = 0; i < 2; ++i) a2[i] = (b2 ? a4[i + 2] : a4[i]) + __shfl_xor(b2 ? a4[i] : a4[i + 2], 4, 64);
    a1 = (b1 ? a2[1] : a2[0]) + __shfl_xor(b1 ? a2[0] : a2[1], 2, 64);
    a1 += __shfl_xor(a1, 1, 64);
  }
  float rmax = (P == 2) ? sqrtf(a1) : a1;             // (a missing row has sum 0)
  for (int off = 32; off > 0; off >>= 1) rmax = fmaxf(rmax, __shfl_xor(rmax, off, 64));
  if (lane == 0) rad[m] = rmax * (1.f + kBoundSlack) + 1e-30f;
}

// ---------------------------------------------------------------------------------------------
// Generic 128 x 128 distance tile in float32 vector arithmetic (no MFMA): rows x_i (+ shift), columns y_j,
// dist_p(x_i + shift, y_j) for p = 1 or 2 (p = 0: the dot product x_i . y_j, MATRIX epilogue only), K staged through LDS in 16-dimension slices, 8 x 8 results
// per thread.  Two epilogues:
//   ASSIGN  first column within delta (= the group radius tau) of every row -> atomicMin on a packed
//           (column position, distance bits) word
//   MATRIX  the p-th power of every distance is written to a row-major n_rows x n_cols matrix
//   BOUND   rows and columns are micro-tile centres; a micro-tile pair survives when
//           dist - rho_row - rho_col <= delta (with slack), and then sets the bit of its join tile
enum { kEpiAssign = 0, kEpiBound = 1, kEpiMatrix = 2, kEpiBoundUnits = 3 };

// Units of the two-level bound test (see k_bound_l2_units further down): a padded group's run of micro-tiles, or a
// single micro-tile of the packed tail region.
struct UnitTable {
  const int32_t* first;   // big units: first micro-tile ...
  const int32_t* n;       // ... and number of micro-tiles
  int n_big;              // units 0 .. n_big - 1 are padded groups
  int tail_first;         // unit n_big + i is micro-tile tail_first + i
  int n_units;
};
__device__ __forceinline__ void unit_range(const UnitTable& ut, int u, int& first, int& n) {
  if (u < ut.n_big) { first = ut.first[u]; n = ut.n[u]; }
  else { first = ut.tail_first + (u - ut.n_big); n = 1; }
}

constexpr int kInlineMicroPairs = 8;   // unit pairs with at most this many micro-tile pairs are refined where they are found
struct BoundPairs {
  unsigned long long* list;     // (rl << 48) | (unit of heads << 24) | unit of tails
  unsigned long long* count;    // entries asked for (may exceed cap)
  unsigned long long cap;
};


struct TileDistArgs {
  const void* X; int dtypeX; const int32_t* row_ids; const int32_t* n_rows_dev; int64_t n_rows;
  const void* Y; int dtypeY; const int32_t* col_ids; const int32_t* n_cols_dev; int64_t n_cols;
  const void* shift; int dtype_shift; int r0;     // optional vector added to every row: shift[(r0 + blockIdx.z) * d ...]
  int d;
  unsigned long long* best;                        // ASSIGN
  float* matrix;                                   // MATRIX
  int64_t matrix_rel_stride;                       // MATRIX: relation blockIdx.z writes its n_rows x n_cols block this many floats further on
  int symmetric;                                   // MATRIX with X == Y and no shift: only the blocks on and above the diagonal work, and write both halves
  const float* rad; float delta; uint32_t* bitmap; // BOUND
  int nH, words_per_row, micro_per_bm, micro_per_bn;
  // BOUND with per-relation summaries (the general form): relation blockIdx.z reads rows z * x_rel_rows + i of X and
  // z * y_rel_rows + j of Y (0: one set for all relations); rad_rows: radii of the rows when they differ from the columns'
  int64_t x_rel_rows, y_rel_rows; const float* rad_rows;
  // BOUND on units (L1): rows / columns are unit centres, rad their radii; survivors are refined on the
  // micro-tile summaries below (small pairs on the spot, the others through the list)
  UnitTable ut; BoundPairs bp;
  const float* fine_cent; const float* fine_rad; int64_t n_micro;
};

// L1 bound of one unit pair on its micro-tile pairs: dist_1(c_H + r, c_T) - rho_H - rho_T <= delta, centre
// distances summed over d by the calling lane; `lane_count` lanes starting at `lane0` share the pairs.
__device__ __forceinline__ void refine_unit_pair_l1(const TileDistArgs& a, int rl, int uH, int uT, int lane0, int lane_count) {
  int fH, nHm, fT, nTm;
  unit_range(a.ut, uH, fH, nHm);
  unit_range(a.ut, uT, fT, nTm);
  const int64_t so = (int64_t)(a.r0 + rl) * a.d;
  const int64_t total = (int64_t)nHm * nTm;
  for (int64_t i = lane0; i < total; i += lane_count) {
    const int64_t mH = fH + i / nTm, mT = fT + i % nTm;
    const float rH = a.fine_rad[mH], rT = a.fine_rad[mT];
    if (rH < 0.f || rT < 0.f) continue;
    const float* cH = a.fine_cent + mH * a.d;
    const float* cT = a.fine_cent + mT * a.d;
    float s = 0.f;
    for (int k = 0; k < a.d; ++k) s += fabsf(cH[k] + ld_elem(a.shift, so + k, a.dtype_shift) - cT[k]);
    if (s * (1.f - kBoundSlack) - rH - rT <= a.delta * (1.f + kBoundSlack)) {
      const int tH = (int)(mH / a.micro_per_bm), tT = (int)(mT / a.micro_per_bn);
      uint32_t* w = &a.bitmap[((int64_t)rl * a.nH + tH) * a.words_per_row + (tT >> 5)];
      if (!(*w & (1u << (tT & 31)))) atomicOr(w, 1u << (tT & 31));
    }
  }
}

template <int P, int EPI>
__global__ __launch_bounds__(256) void k_tile_dist(const TileDistArgs a) {
  constexpr int BM = 128, BN = 128, BK = 16;
  __shared__ __attribute__((aligned(16))) float As[BK][BM];
  __shared__ __attribute__((aligned(16))) float Bs[BK][BN];
  __shared__ int32_t rid[BM], cid[BN];
  const int tid = threadIdx.x;
  const int64_t n_rows = a.n_rows_dev ? (int64_t)*a.n_rows_dev : a.n_rows;
  const int64_t n_cols = a.n_cols_dev ? (int64_t)*a.n_cols_dev : a.n_cols;
  const int64_t row0 = (int64_t)blockIdx.y * BM, col0 = (int64_t)blockIdx.x * BN;
  if (row0 >= n_rows || col0 >= n_cols) return;
  if (EPI == kEpiMatrix && a.symmetric && blockIdx.y > blockIdx.x) return;      // the mirror block writes this one
  if (tid < BM) {
    const int64_t r = row0 + tid;
    rid[tid] = r < n_rows ? (a.row_ids ? a.row_ids[r] : (int32_t)r) : -1;
  } else {
    const int64_t c = col0 + (tid - BM);
    cid[tid - BM] = c < n_cols ? (a.col_ids ? a.col_ids[c] : (int32_t)c) : -1;
  }
  __syncthreads();
  const int d = a.d;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  const int srow = tid >> 1, sk0 = (tid & 1) * 8;
  const int re = rid[srow], ce = cid[srow];
  const int64_t xo = ((int64_t)blockIdx.z * a.x_rel_rows + (re < 0 ? 0 : re)) * d,
                yo = ((int64_t)blockIdx.z * a.y_rel_rows + (ce < 0 ? 0 : ce)) * d;
  const int64_t so = (int64_t)(a.r0 + (int)blockIdx.z) * d;
  for (int k0 = 0; k0 < d; k0 += BK) {
    float va[8], vb[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int k = k0 + sk0 + q;
      const bool in = k < d;
      float x = in ? ld_elem(a.X, xo + k, a.dtypeX) : 0.f;
      if (in && a.shift) x += ld_elem(a.shift, so + k, a.dtype_shift);
      va[q] = x;
      vb[q] = in ? ld_elem(a.Y, yo + k, a.dtypeY) : 0.f;
    }
    __syncthreads();
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
        for (int j = 0; j < 8; ++j) {
          if (P == 0) {
            acc[i][j] += av[i] * bv[j];
          } else {
            const float x = av[i] - bv[j];
            acc[i][j] += (P == 2) ? x * x : fabsf(x);
          }
        }
    }
  }
  // rows of this thread: (i >> 2) * 64 + ty * 4 + (i & 3); columns: (j >> 2) * 64 + tx * 4 + (j & 3)
  if (EPI == kEpiAssign) {
    // Among the columns (pivots) within tau of the row, the one with the LOWEST position wins, not the
    // nearest: when a natural cluster received several pivots, all its rows then agree on one of them
    // instead of splitting the cluster between them.
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int lr = (i >> 2) * 64 + ty * 4 + (i & 3);
      unsigned long long bestv = ~0ull;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int lc = (j >> 2) * 64 + tx * 4 + (j & 3);
        const float dist = (P == 2) ? sqrtf(acc[i][j]) : acc[i][j];
        if (cid[lc] >= 0 && dist <= a.delta) {
          const unsigned long long v =
              ((unsigned long long)(uint32_t)(col0 + lc) << 32) | (unsigned long long)__float_as_uint(dist);
          bestv = v < bestv ? v : bestv;
        }
      }
      // the 16 threads that share a row are 16 consecutive lanes
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)(bestv & 0xffffffffull), off, 16);
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(bestv >> 32), off, 16);
        const unsigned long long o = ((unsigned long long)hi << 32) | lo;
        bestv = o < bestv ? o : bestv;
      }
      if (tx == 0 && rid[lr] >= 0 && bestv != ~0ull) atomicMin(&a.best[row0 + lr], bestv);
    }
  } else if (EPI == kEpiMatrix) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int lr = (i >> 2) * 64 + ty * 4 + (i & 3);
      if (rid[lr] < 0) continue;
#pragma unroll
      for (int jg = 0; jg < 2; ++jg) {
        const int lc = jg * 64 + tx * 4;
        float* o = a.matrix + (int64_t)blockIdx.z * a.matrix_rel_stride + (row0 + lr) * n_cols + col0 + lc;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (cid[lc + j] >= 0) o[j] = acc[i][jg * 4 + j];
        if (a.symmetric && blockIdx.y != blockIdx.x) {       // sum of (x_i - x_j)^2 = sum of (x_j - x_i)^2, term by term
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (cid[lc + j] >= 0) a.matrix[(int64_t)blockIdx.z * a.matrix_rel_stride + (col0 + lc + j) * n_cols + row0 + lr] = acc[i][jg * 4 + j];
        }
      }
    }
  } else if (EPI == kEpiBoundUnits) {
    const int rl = (int)blockIdx.z;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int lr = (i >> 2) * 64 + ty * 4 + (i & 3);
      if (rid[lr] < 0) continue;
      const float rr = a.rad[row0 + lr];
      if (rr < 0.f) continue;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int lc = (j >> 2) * 64 + tx * 4 + (j & 3);
        if (cid[lc] < 0) continue;
        const float rc = a.rad[col0 + lc];
        if (rc < 0.f) continue;
        const float dist = (P == 2) ? sqrtf(acc[i][j]) : acc[i][j];
        if (dist * (1.f - kBoundSlack) - rr - rc > a.delta * (1.f + kBoundSlack)) continue;
        const int uH = (int)(row0 + lr), uT = (int)(col0 + lc);
        int fH, nHm, fT, nTm;
        unit_range(a.ut, uH, fH, nHm);
        unit_range(a.ut, uT, fT, nTm);
        unsigned long long pos = a.bp.cap;
        if ((int64_t)nHm * nTm > kInlineMicroPairs) pos = atomicAdd(a.bp.count, 1ull);
        if (pos < a.bp.cap)
          a.bp.list[pos] = ((unsigned long long)(uint32_t)rl << 48) | ((unsigned long long)(uint32_t)uH << 24) |
                           (unsigned long long)(uint32_t)uT;
        else
          refine_unit_pair_l1(a, rl, uH, uT, 0, 1);
      }
    }
  } else {
    const int rl = (int)blockIdx.z;
    const float* rad_r = (a.rad_rows ? a.rad_rows : a.rad) + (int64_t)rl * a.x_rel_rows;
    const float* rad_c = a.rad + (int64_t)rl * a.y_rel_rows;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int lr = (i >> 2) * 64 + ty * 4 + (i & 3);
      if (rid[lr] < 0) continue;
      const float rr = rad_r[row0 + lr];
      if (rr < 0.f) continue;                                  // empty micro-tile
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int lc = (j >> 2) * 64 + tx * 4 + (j & 3);
        if (cid[lc] < 0) continue;
        const float rc = rad_c[col0 + lc];
        if (rc < 0.f) continue;
        const float dist = (P == 2) ? sqrtf(acc[i][j]) : acc[i][j];
        const float lb = dist * (1.f - kBoundSlack) - rr - rc;  // radii already carry their slack
        if (lb <= a.delta * (1.f + kBoundSlack)) {
          const int tH = (int)((row0 + lr) / a.micro_per_bm), tT = (int)((col0 + lc) / a.micro_per_bn);
          atomicOr(&a.bitmap[((int64_t)rl * a.nH + tH) * a.words_per_row + (tT >> 5)], 1u << (tT & 31));
        }
      }
    }
  }
}

// The same MATRIX results for small operands (a few hundred to a few thousand rows and columns: micro-tile centres,
// relation vectors), where the 128 x 128 tiles above leave most of the chip idle: 32 x 32 results per block of 256
// threads, K through LDS 128 dimensions at a time, four rows x one column per thread.  out[i][j] = ||x_i - y_j||^2
// (P = 2) or x_i . y_j (P = 0), row-major n_rows x n_cols; X rows of the given type, Y rows float32.
// With `rad` set (P = 2, X = Y = the micro-tile centres) the result is not the squared centre distance D itself but
// the part of the flat bound test that depends on the pair alone, reach^2 (1 + slack) + D (d + 8) 2^-24 - D with
// reach = delta (1 + slack) + rad_i + rad_j (see k_bound_l2), so that the test does not form it again for every
// group of relations; a pair with an empty micro-tile (rad < 0) gets -3e38 and never passes.
template <int P>
__global__ __launch_bounds__(256) void k_small_matrix(const void* __restrict__ X, int dtypeX, int64_t n_rows,
                                                      const float* __restrict__ Y, int64_t n_cols, int d,
                                                      float* __restrict__ out, const float* __restrict__ rad = nullptr,
                                                      float delta = 0.f, int symmetric = 0) {      // symmetric (X == Y): blocks above the diagonal write both halves
  constexpr int KC = 128;                                 // dimensions per pass through LDS (d <= 128: one pass, two barriers)
  __shared__ float xs[32][KC + 1], ys[32][KC + 1];
  const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
  const int64_t row0 = (int64_t)blockIdx.y * 32, col0 = (int64_t)blockIdx.x * 32;
  if (symmetric && blockIdx.y > blockIdx.x) return;        // the mirror block writes this one
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < d; k0 += KC) {
    const int kn = d - k0 < KC ? d - k0 : KC;
    __syncthreads();
    // 32 rows x kn dimensions of each operand, consecutive threads on consecutive dimensions of a row
    for (int e = tid; e < 32 * KC; e += 256) {
      const int rw = e / KC, k = e - rw * KC;
      const bool in = k < kn;
      xs[rw][k] = (in && row0 + rw < n_rows) ? ld_elem(X, (row0 + rw) * d + k0 + k, dtypeX) : 0.f;
      ys[rw][k] = (in && col0 + rw < n_cols) ? Y[(col0 + rw) * d + k0 + k] : 0.f;
    }
    __syncthreads();
    for (int k = 0; k < kn; ++k) {
      const float b = ys[tx][k];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = xs[ty + 8 * q][k];
        if (P == 0) acc[q] += a * b;
        else { const float x = a - b; acc[q] += x * x; }
      }
    }
  }
  if (col0 + tx < n_cols) {
    const float rT = rad ? rad[col0 + tx] : 0.f;
    const float dsl = delta * (1.f + kBoundSlack), dk = (float)(d + 8) * 6e-8f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (row0 + ty + 8 * q < n_rows) {
        float v = acc[q];
        if (rad) {
          const float rH = rad[row0 + ty + 8 * q];
          const float reach = dsl + (rH + rT);                 // (the same for both orders of the pair)
          v = (rH < 0.f || rT < 0.f) ? -3e38f : reach * reach * (1.f + kBoundSlack) + v * dk - v;
        }
        out[(row0 + ty + 8 * q) * n_cols + col0 + tx] = v;
        if (symmetric && blockIdx.y != blockIdx.x) out[(col0 + tx) * n_cols + row0 + ty + 8 * q] = v;   // (sum of (x_i - x_j)^2 = sum of (x_j - x_i)^2 term by term, and the pair term is symmetric too)
      }
  }
}

// out[i][j] = x_i . y_j for small operands, on the float32 matrix pipes: one wave per 32 x 32 results, no LDS and no
// barrier.  v_mfma_f32_32x32x2_f32 takes A[i][k] from lane 32 k + i and B[k][j] from lane 32 k + j (k = 0, 1); a dot
// product does not care in which order its dimensions are taken as long as both operands agree, so lane (row, half)
// reads the four consecutive elements 8 g + 4 half .. + 3 of its row in one load and feeds them to four successive
// steps.  All loads of up to 128 dimensions are issued before the first is used: a chunk costs one memory round trip.
// Products and sums are float32 (the bound test charges (d + 8) 2^-24 ||x|| ||y|| for them, which holds for any order
// of a float32 sum of d products).  X rows of the given storage type, Y rows float32; VEC: rows may be read four
// elements at a time (both bases on 16-byte boundaries -- 8 for bf16 rows -- and d a multiple of four).
template <bool BF16, bool VEC>
__global__ __launch_bounds__(64) void k_small_dot(const void* __restrict__ X, int64_t n_rows, const float* __restrict__ Y,
                                                  int64_t n_cols, int d, float* __restrict__ out) {
  const int lane = threadIdx.x, row = lane & 31, half = lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.y * 32, col0 = (int64_t)blockIdx.x * 32;
  const int64_t xr = row0 + row < n_rows ? row0 + row : n_rows - 1;      // (past the end: a valid row, the results are dropped)
  const int64_t yc = col0 + row < n_cols ? col0 + row : n_cols - 1;
  const int64_t xo = xr * d, yo = yc * d;
  f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  constexpr int kG = 16;                                                  // groups of 8 dimensions per chunk (d <= 128: one chunk)
  for (int k0 = 0; k0 < d; k0 += 8 * kG) {
    f32x4_t xv[kG], yv[kG];
#pragma unroll
    for (int g = 0; g < kG; ++g) {
      const int k = k0 + 8 * g + 4 * half;
      xv[g] = exact_ld4<BF16, VEC>(X, xo, k, d);
      yv[g] = exact_ld4<false, VEC>(Y, yo, k, d);
    }
    __builtin_amdgcn_sched_barrier(0);                                    // (the loads stay together, ahead of the arithmetic)
#pragma unroll
    for (int g = 0; g < kG; ++g) {
      if (k0 + 8 * g >= d) break;                                         // the same for the whole wave
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xv[g][e], yv[g][e], acc, 0, 0, 0);
    }
  }
  // register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
  if (col0 + row < n_cols) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t i = row0 + 8 * (v >> 2) + 4 * half + (v & 3);
      if (i < n_rows) out[i * n_cols + col0 + row] = acc[v];
    }
  }
}

// L2 only.  u[rl][m] = r . c_m and rn[rl] = ||r||^2 for the relations of a batch: one wave per (rl, m).
__global__ __launch_bounds__(256) void k_rel_centre_dot(const void* __restrict__ Rv, int dtype, int d, int r0, int RB,
                                                        const float* __restrict__ cent, int64_t n_micro,
                                                        float* __restrict__ u, float* __restrict__ rn) {
  const int lane = threadIdx.x & 63;
  const int64_t w = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t per_rel = n_micro + 1;                       // the extra item computes ||r||^2
  if (w >= per_rel * RB) return;
  const int rl = (int)(w / per_rel);
  const int64_t m = w - (int64_t)rl * per_rel;
  const int64_t ro = (int64_t)(r0 + rl) * d;
  float s = 0.f;
  if (m == n_micro) {
    for (int k = lane; k < d; k += 64) { const float x = ld_elem(Rv, ro + k, dtype); s += x * x; }
  } else {
    const float* c = cent + m * d;
    for (int k = lane; k < d; k += 64) s += ld_elem(Rv, ro + k, dtype) * c[k];
  }
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (lane == 0) {
    if (m == n_micro) rn[rl] = s; else u[(int64_t)rl * n_micro + m] = s;
  }
}

// L2 only.  The squared centre distance of a micro-tile pair under relation r expands into parts that do
// not need a d-dimensional loop per (r, H, T):
//     ||c_H + r - c_T||^2 = ||c_H - c_T||^2 + 2 (r.c_H - r.c_T) + ||r||^2 = D[H][T] + 2 (u[r][H] - u[r][T]) + rn[r]
// (the same observation that makes distB independent of r in Section 5.2, applied to the bound).  The float32 cancellation error of the sum is bounded by
// err = 2 (d + 8) 2^-24 ||r|| (||c_H|| + ||c_T||) + (d + 8) 2^-24 D and added on the keeping side: D itself is a float32
// sum of d squared differences (relative error at most (d + 4) 2^-24 in the worst case), and for TransE data it is far
// larger than reach^2 (r cancels c_H - c_T), so its error is charged in full, not absorbed in the slack of reach^2.
constexpr int kRelChunk = 16;
struct BoundL2Args {
  const float* D; const float* u; const float* rn; const float* rad; const float* cnorm;
  int64_t n_micro; int RB; int d; float delta;
  uint32_t* bitmap; int nH, words_per_row, micro_per_bm, micro_per_bn;
  // micro-tile level of the two-level test without the D and u matrices (D == NULL): centre distances are then
  // summed directly from the centres and the relation vector
  const float* cent; const void* Rv; int dtype; int r0;
  // k_bound_l2 only, optional (NULL: off): every tile whose bit is set for the first time is also appended to a flat
  // list -- its tail tile to list_cols, its row (relation, head tile) to list_rows and to list_active -- so that a
  // batch with few surviving tiles needs no pass over the bitmap (see k_batch_tiles)
  uint32_t* list_cols; uint32_t* list_rows; uint32_t* list_active; unsigned long long* list_count; unsigned long long list_cap;
};
constexpr int kHeadChunk = 16;
constexpr int kHeadsFlat = 64;       // head micro-tiles per block of the flat test (four groups of kHeadChunk)
// PAIR_READY: a.D holds the pair's part of the right side, ready made (k_small_matrix with radii), not the plain
// squared centre distance: a test then costs one load, one addition and one comparison.
// UNITS: the unit level of the two-level test (see below): `a` describes UNITS, and a surviving (relation, unit pair)
// is appended to the list `bp` -- or refined on the spot on the micro-tile arrays `fine` when the pair is small or
// the list is full -- instead of setting bits.
template <bool LIST>
__device__ __forceinline__ void refine_unit_pair(const BoundL2Args& a, const UnitTable& ut, int rl, int uH, int uT, int lane0,
                                                 int lane_count);
// The surviving (relation rl0 + q, unit pair) of a wave: bit q of `keep` per lane (head unit mH the same for the wave,
// tail unit mT the lane's).  A pair of small units (in the packed tail region both are single micro-tiles) is
// finished on the spot; pairs with many micro-tile pairs go through the list, whose length is advanced ONCE per
// relation for all lanes of the wave that append (atomics on one address are served one after the other: with one
// per entry the unit level of a join with many survivors spent most of its time there).  Called by all active lanes.
template <bool LIST>
__device__ __forceinline__ void unit_pairs_out(uint32_t keep, int rl0, int mH, int mT, const BoundL2Args& fine,
                                               const UnitTable& ut, const BoundPairs& bp) {
  if (__builtin_amdgcn_ballot_w64(keep != 0u) == 0ull) return;
  int fH, nHm, fT, nTm;
  unit_range(ut, mH, fH, nHm);
  unit_range(ut, mT, fT, nTm);
  // (without the matrices a micro-tile pair costs a loop over d: then every pair but a single one is listed)
  const bool big = (int64_t)nHm * nTm > (fine.D ? kInlineMicroPairs : 1);
  const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
#pragma unroll 1
  for (int q = 0; q < kRelChunk; ++q) {
    const bool k = (keep >> q) & 1u;
    if (__builtin_amdgcn_ballot_w64(k) == 0ull) continue;
    const unsigned long long ml = __builtin_amdgcn_ballot_w64(k && big);
    unsigned long long pos = bp.cap;
    if (ml) {
      const int leader = (int)__builtin_ctzll(ml);
      unsigned long long base = 0ull;
      if (lane == leader) base = atomicAdd(bp.count, (unsigned long long)__builtin_popcountll(ml));
      const uint32_t blo = (uint32_t)__shfl((int)(uint32_t)(base & 0xffffffffull), leader, 64);
      const uint32_t bhi = (uint32_t)__shfl((int)(uint32_t)(base >> 32), leader, 64);
      if (k && big) pos = (((unsigned long long)bhi << 32) | blo) + (unsigned long long)__builtin_popcountll(ml & ((1ull << lane) - 1ull));
    }
    if (k) {
      if (pos < bp.cap)
        bp.list[pos] = ((unsigned long long)(uint32_t)(rl0 + q) << 48) | ((unsigned long long)(uint32_t)mH << 24) |
                       (unsigned long long)(uint32_t)mT;
      else
        refine_unit_pair<LIST>(fine, ut, rl0 + q, mH, mT, 0, 1);
    }
  }
}
// LIST (UNITS only): the micro-tile level also lists the tiles it keeps (see keep_tile)
template <bool PAIR_READY, bool UNITS, bool LIST = false>
__global__ __launch_bounds__(256) void k_bound_l2(const BoundL2Args a, const BoundL2Args fine, const UnitTable ut,
                                                  const BoundPairs bp) {
  // block = 256 tail micro-tiles x kHeadsFlat head micro-tiles x kRelChunk relations; the per-(head, relation)
  // terms sit in LDS, the thread's own per-relation terms in registers, so one test costs one (shared) D load per
  // kRelChunk relations, one addition and one comparison -- and most chunks of relations end at one comparison
  __shared__ __attribute__((aligned(16))) float aH[kHeadsFlat][kRelChunk];   // 2 r.c_H + ||r||^2 - kk ||c_H|| ||r|| per (head micro-tile, relation)
  __shared__ float srnS[kRelChunk];
  __shared__ float radH[kHeadsFlat], aHmin[kHeadsFlat];
  const int tid = threadIdx.x;
  const int64_t mT = (int64_t)blockIdx.x * blockDim.x + tid;
  const int64_t mH0 = (int64_t)blockIdx.y * kHeadsFlat;
  const int rl0 = (int)blockIdx.z * kRelChunk;
  const float kk = 2.f * (float)(a.d + 12) * 6e-8f;
  {
    // 256 threads = kRelChunk relations x 16 neighbouring heads per pass: a row of u is read 64 bytes at a time (one
    // thread per relation and sixteenth of the heads would pull a whole cache line per value: 64 lines per load
    // instruction, 0.4 GB through the vector caches per launch for a matrix of 4 MB)
    const int q = tid >> 4, j = tid & 15;
    const int rl = rl0 + q;
    const float rnq = rl < a.RB ? a.rn[rl] : 0.f;
    const float srn = sqrtf(rnq);
#pragma unroll
    for (int pass = 0; pass < kHeadsFlat / 16; ++pass) {
      const int hq = pass * 16 + j;
      const int64_t mH = mH0 + hq;
      const bool in = rl < a.RB && mH < a.n_micro;
      const float ah = in ? 2.f * a.u[(int64_t)rl * a.n_micro + mH] + rnq * (1.f - 2.4e-7f) : 0.f;
      aH[hq][q] = in ? ah - (kk * a.cnorm[mH]) * srn : 0.f;
    }
    if (tid < kRelChunk) srnS[tid] = sqrtf(rl0 + tid < a.RB ? a.rn[rl0 + tid] : 0.f);
    if (tid < kHeadsFlat) {
      const int64_t m = mH0 + tid;
      radH[tid] = m < a.n_micro ? a.rad[m] : -1.f;
    }
  }
  __syncthreads();
  {
    // the smallest left side of every head micro-tile over the chunk's relations: four threads per head
    const int hq = tid >> 2, part = tid & 3;
    float mn = 3e38f;
    if (mH0 + hq < a.n_micro) {
#pragma unroll
      for (int i = 0; i < 4; ++i) mn = rl0 + part * 4 + i < a.RB ? fminf(mn, aH[hq][part * 4 + i]) : mn;
    }
    mn = fminf(mn, __shfl_xor(mn, 1, 64));
    mn = fminf(mn, __shfl_xor(mn, 2, 64));
    if (part == 0) aHmin[hq] = mn;
  }
  __syncthreads();
  if (mT >= a.n_micro) return;
  const float rT = a.rad[mT];
  if (rT < 0.f) return;                                          // empty micro-tile
  const float cT = a.cnorm[mT];
  const int heads_here = a.n_micro - mH0 < kHeadsFlat ? (int)(a.n_micro - mH0) : kHeadsFlat;
  // dist^2 <= lim + ek sqrt(rn), ek = kk (||c_H|| + ||c_T||)
  //   <=>   (2 u_H + rn) - kk ||c_H|| sqrt(rn)  <=  (lim - D) + (2 u_T + kk ||c_T|| sqrt(rn)):
  // the left side is formed once per (head micro-tile, relation) and block, the last term once per (thread, relation),
  // lim - D once per micro-tile pair, which leaves one addition and one comparison per test.  The extra roundings of
  // this order (two each at most 2^-24 of |2 u_H + rn| and of |2 u_T|, three of D) are paid for on the keeping side:
  // 4 more units in the (d + 8) factor of ek, 2.4e-7 of rn and of D.
  float bT[kRelChunk];
  const int nrel = a.RB - rl0 < kRelChunk ? a.RB - rl0 : kRelChunk;
#pragma unroll
  for (int q = 0; q < kRelChunk; ++q)
    bT[q] = q < nrel ? 2.f * a.u[(int64_t)(rl0 + q) * a.n_micro + mT] + (kk * cT) * srnS[q] : -3e38f;   // past the batch: never passes
  // One comparison first for the whole chunk: no relation can pass when even the smallest left side exceeds the right
  // side with the largest per-relation term (float addition is monotonic, so this is the 16 tests' own arithmetic:
  // nothing is widened).  For TransE data the two sides are 6 sigma apart, so almost every chunk ends here.
  float bmax = bT[0];
#pragma unroll
  for (int q = 1; q < kRelChunk; ++q) bmax = fmaxf(bmax, bT[q]);
  const int tT = UNITS ? 0 : (int)(mT / a.micro_per_bn);
  const float dsl = a.delta * (1.f + kBoundSlack);
  const float dk = (float)(a.d + 8) * 6e-8f;
  for (int hg = 0; hg < kHeadsFlat; hg += kHeadChunk) {
  if (mH0 + hg >= a.n_micro) break;                              // the same for the block
  // the centre distances of a group of heads, all loads in flight together (a head past the end reads the group's first row; it is skipped below)
  float Dv[kHeadChunk];
  {
    const float* Dp = a.D + (mH0 + hg) * a.n_micro + mT;
    const int nvalid = a.n_micro - (mH0 + hg) < kHeadChunk ? (int)(a.n_micro - (mH0 + hg)) : kHeadChunk;
#pragma unroll
    for (int hq = 0; hq < kHeadChunk; ++hq) Dv[hq] = Dp[hq < nvalid ? (int64_t)hq * a.n_micro : 0];
  }
#pragma unroll
  for (int hl = 0; hl < kHeadChunk; ++hl) {
    const int hq = hg + hl;
    float rhs;
    if (PAIR_READY) {
      if (hq >= heads_here) break;                               // past the end (the same for the block)
      rhs = Dv[hl];                                              // (-3e38 for an empty micro-tile)
    } else {
      const float rH = radH[hq];
      if (rH < 0.f) continue;                                    // empty or past the end
      const float D = Dv[hl];
      const float reach = dsl + rH + rT;
      rhs = reach * reach * (1.f + kBoundSlack) + D * dk - D;
    }
    const int64_t mH = mH0 + hq;
    if (__builtin_amdgcn_ballot_w64(aHmin[hq] <= rhs + bmax) == 0ull) continue;
    bool any = false;
#pragma unroll
    for (int q = 0; q < kRelChunk; ++q) any |= aH[hq][q] <= rhs + bT[q];
    if (__builtin_amdgcn_ballot_w64(any) == 0ull) continue;      // almost always: nothing survives
    uint32_t keep = 0u;
#pragma unroll
    for (int q = 0; q < kRelChunk; ++q) keep |= (aH[hq][q] <= rhs + bT[q]) ? (1u << q) : 0u;
    if constexpr (UNITS) {
      unit_pairs_out<LIST>(keep, rl0, (int)mH, (int)mT, fine, ut, bp);
      continue;
    }
    const int tH = (int)(mH / a.micro_per_bm);
    while (keep) {
      const int q = __builtin_ctz(keep);
      keep &= keep - 1u;
      const int64_t row = (int64_t)(rl0 + q) * a.nH + tH;
      const uint32_t bit = 1u << (tT & 31);
      const uint32_t old = atomicOr(&a.bitmap[row * a.words_per_row + (tT >> 5)], bit);
      if (a.list_count && !(old & bit)) {                        // the tile is new: also onto the flat list
        const unsigned long long idx = atomicAdd(a.list_count, 1ull);
        if (idx < a.list_cap) { a.list_cols[idx] = (uint32_t)tT; a.list_rows[idx] = (uint32_t)row; a.list_active[idx] = (uint32_t)row; }
      }
    }
  }
  }   // groups of heads
}

// ---------------------------------------------------------------------------------------------
// Two-level bound test (L2).  When groups span several micro-tiles, the flat test over micro-tile pairs does
// the same work many times: all micro-tiles of a group sit within the group's radius of one another.  A
// UNIT is a padded group (its run of micro-tiles) or, in the packed tail region, a single micro-tile.  The
// same bound is first taken on unit pairs -- centre = mean of the micro-tile centres, radius = max over
// the micro-tiles of (distance of its centre to the unit centre + its radius), so every row of the unit is
// inside -- and only the micro-tile pairs of surviving unit pairs are tested.  Survivors go through a list;
// a lane that finds the list full tests its pair's micro-tiles on the spot.
// one wave per unit; P: the join's metric (radii in that metric)
template <int P>
__global__ __launch_bounds__(64) void k_unit_summary(const float* __restrict__ cent, const float* __restrict__ rad, int d,
                                                     UnitTable ut, float* __restrict__ centU, float* __restrict__ radU,
                                                     float* __restrict__ cnormU) {
  const int u = (int)blockIdx.x;
  if (u >= ut.n_units) return;
  const int lane = threadIdx.x;
  int first, n;
  unit_range(ut, u, first, n);
  int cntm = 0;
  for (int m = first; m < first + n; ++m) cntm += rad[m] >= 0.f;
  float* c = centU + (int64_t)u * d;
  if (cntm == 0) {
    for (int k = lane; k < d; k += 64) c[k] = 0.f;
    if (lane == 0) { radU[u] = -1.f; cnormU[u] = 0.f; }
    return;
  }
  const float inv = 1.f / (float)cntm;
  float c2 = 0.f;
  for (int k = lane; k < d; k += 64) {
    float s = 0.f;
    for (int m = first; m < first + n; ++m)
      if (rad[m] >= 0.f) s += cent[(int64_t)m * d + k];
    c[k] = s * inv;
    c2 += (s * inv) * (s * inv);
  }
  for (int off = 32; off > 0; off >>= 1) c2 += __shfl_xor(c2, off, 64);
  __syncthreads();
  float rmax = 0.f;
  for (int m = first; m < first + n; ++m) {
    if (rad[m] < 0.f) continue;
    float s = 0.f;
    for (int k = lane; k < d; k += 64) { const float x = cent[(int64_t)m * d + k] - c[k]; s += (P == 2) ? x * x : fabsf(x); }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    rmax = fmaxf(rmax, ((P == 2) ? sqrtf(s) : s) * (1.f + kBoundSlack) + rad[m]);
  }
  if (lane == 0) { radU[u] = rmax * (1.f + kBoundSlack) + 1e-30f; cnormU[u] = sqrtf(c2) * (1.f + kBoundSlack); }
}

// the micro-tile level of the test for one surviving unit pair and relation; `lane_count` lanes starting at
// `lane0` share the micro-tile pairs (1 lane = on the spot in the unit-level kernel, a block in k_bound_refine)
// a surviving join tile: its bit in the bitmap, and -- LIST: the first time -- its entry on the flat list (see
// k_batch_tiles).  A template parameter and not a test of a.list_count: with both forms in one kernel the atomic of the
// plain form became a returning one too, and a join with many surviving tiles (N = 1,000,000) lost a third of its
// bound test's speed.
template <bool LIST>
__device__ __forceinline__ void keep_tile(const BoundL2Args& a, int rl, int tH, int tT) {
  const int64_t row = (int64_t)rl * a.nH + tH;
  uint32_t* w = &a.bitmap[row * a.words_per_row + (tT >> 5)];
  const uint32_t bit = 1u << (tT & 31);
  if (*w & bit) return;                                          // (most micro-tile pairs of a tile find it set)
  if constexpr (!LIST) {
    atomicOr(w, bit);
  } else {
    const uint32_t old = atomicOr(w, bit);
    if (!(old & bit)) {
      const unsigned long long idx = atomicAdd(a.list_count, 1ull);
      if (idx < a.list_cap) { a.list_cols[idx] = (uint32_t)tT; a.list_rows[idx] = (uint32_t)row; a.list_active[idx] = (uint32_t)row; }
    }
  }
}
template <bool LIST>
__device__ __forceinline__ void refine_unit_pair(const BoundL2Args& a, const UnitTable& ut, int rl, int uH, int uT, int lane0,
                                                 int lane_count) {
  int fH, nHm, fT, nTm;
  unit_range(ut, uH, fH, nHm);
  unit_range(ut, uT, fT, nTm);
  const float rnq = a.rn[rl], srn = sqrtf(rnq);
  const float dsl = a.delta * (1.f + kBoundSlack);
  const float kk = 2.f * (float)(a.d + 12) * 6e-8f;
  const int64_t total = (int64_t)nHm * nTm;
  for (int64_t i = lane0; i < total; i += lane_count) {
    const int64_t mH = fH + i / nTm, mT = fT + i % nTm;
    const float rH = a.rad[mH], rT = a.rad[mT];
    if (rH < 0.f || rT < 0.f) continue;
    if (!a.D) {           // small problems: no matrices, the distance of c_H + r and c_T summed over d
      const float* cH = a.cent + mH * a.d;
      const float* cT = a.cent + mT * a.d;
      const int64_t so = (int64_t)(a.r0 + rl) * a.d;
      float sq = 0.f;
      for (int k = 0; k < a.d; ++k) {
        const float x = cH[k] + ld_elem(a.Rv, so + k, a.dtype) - cT[k];
        sq += x * x;
      }
      if (sqrtf(sq) * (1.f - kBoundSlack) - rH - rT <= dsl) keep_tile<LIST>(a, rl, (int)(mH / a.micro_per_bm), (int)(mT / a.micro_per_bn));
      continue;
    }
    const float D = a.D[mH * a.n_micro + mT];
    const float reach = dsl + rH + rT;
    const float rhs = reach * reach * (1.f + kBoundSlack) + D * ((float)(a.d + 8) * 6e-8f) - D;
    const float ek = kk * (a.cnorm[mH] + a.cnorm[mT]);
    const float lhs = (2.f * a.u[(int64_t)rl * a.n_micro + mH] + rnq * (1.f - 2.4e-7f)) - 2.f * a.u[(int64_t)rl * a.n_micro + mT] -
                      ek * srn;
    if (lhs <= rhs) keep_tile<LIST>(a, rl, (int)(mH / a.micro_per_bm), (int)(mT / a.micro_per_bn));
  }
}

// Unit level: the flat kernel's arithmetic on unit summaries (a.D, a.u, a.rad, a.cnorm and a.n_micro then
// describe UNITS); survivors are appended to the list, or refined on the spot when the list is full.
// `fine` holds the micro-tile level arrays for that case.
template <bool LIST>
__global__ __launch_bounds__(256) void k_bound_l2_units(const BoundL2Args a, const BoundL2Args fine, const UnitTable ut,
                                                        const BoundPairs bp) {
  __shared__ float aH[kHeadChunk][kRelChunk];
  __shared__ float srnS[kRelChunk];
  __shared__ float radH[kHeadChunk], cnH[kHeadChunk];
  const int tid = threadIdx.x;
  const int64_t mT = (int64_t)blockIdx.x * blockDim.x + tid;
  const int64_t mH0 = (int64_t)blockIdx.y * kHeadChunk;
  const int rl0 = (int)blockIdx.z * kRelChunk;
  {
    const int q = tid / kHeadChunk, hq = tid % kHeadChunk;      // neighbouring threads on neighbouring heads: 64 bytes of a row of u
    const int rl = rl0 + q;
    const int64_t mH = mH0 + hq;
    const float rnq = rl < a.RB ? a.rn[rl] : 0.f;
    aH[hq][q] = (rl < a.RB && mH < a.n_micro) ? 2.f * a.u[(int64_t)rl * a.n_micro + mH] + rnq * (1.f - 2.4e-7f) : 0.f;
    if (tid < kRelChunk) srnS[tid] = sqrtf((rl0 + tid < a.RB) ? a.rn[rl0 + tid] : 0.f);
    if (tid < kHeadChunk) {
      const int64_t m = mH0 + tid;
      radH[tid] = m < a.n_micro ? a.rad[m] : -1.f;
      cnH[tid] = m < a.n_micro ? a.cnorm[m] : 0.f;
    }
  }
  __syncthreads();
  if (mT >= a.n_micro) return;
  const float rT = a.rad[mT];
  if (rT < 0.f) return;
  const float cT = a.cnorm[mT];
  float bT[kRelChunk];
  const int nrel = a.RB - rl0 < kRelChunk ? a.RB - rl0 : kRelChunk;
#pragma unroll
  for (int q = 0; q < kRelChunk; ++q) bT[q] = q < nrel ? 2.f * a.u[(int64_t)(rl0 + q) * a.n_micro + mT] : -3e38f;
  const float dsl = a.delta * (1.f + kBoundSlack);
  const float kk = 2.f * (float)(a.d + 12) * 6e-8f;
  // the centre distances of the block's heads, all loads in flight together (a head past the end reads the first row; it is skipped below)
  float Dv[kHeadChunk];
  {
    const float* Dp = a.D + mH0 * a.n_micro + mT;
    const int nvalid = a.n_micro - mH0 < kHeadChunk ? (int)(a.n_micro - mH0) : kHeadChunk;
#pragma unroll
    for (int hq = 0; hq < kHeadChunk; ++hq) Dv[hq] = Dp[hq < nvalid ? (int64_t)hq * a.n_micro : 0];
  }
#pragma unroll
  for (int hq = 0; hq < kHeadChunk; ++hq) {
    const float rH = radH[hq];
    if (rH < 0.f) continue;
    const int64_t mH = mH0 + hq;
    const float D = Dv[hq];
    const float reach = dsl + rH + rT;
    const float rhs = reach * reach * (1.f + kBoundSlack) + D * ((float)(a.d + 8) * 6e-8f) - D;
    const float ek = kk * (cnH[hq] + cT);
    uint32_t keep = 0u;
#pragma unroll
    for (int q = 0; q < kRelChunk; ++q) keep |= (aH[hq][q] - bT[q] - ek * srnS[q] <= rhs) ? (1u << q) : 0u;
    unit_pairs_out<LIST>(keep, rl0, (int)mH, (int)mT, fine, ut, bp);
  }
}

// L1 form of k_bound_refine (below): the listed unit pairs on their micro-tile summaries.
__global__ __launch_bounds__(256) void k_bound_refine_l1(const TileDistArgs a) {
  const unsigned long long n = *a.bp.count < a.bp.cap ? *a.bp.count : a.bp.cap;
  for (unsigned long long e = blockIdx.x; e < n; e += gridDim.x) {
    const unsigned long long v = a.bp.list[e];
    refine_unit_pair_l1(a, (int)(v >> 48), (int)((v >> 24) & 0xffffffull), (int)(v & 0xffffffull),
                        (int)(blockIdx.y * blockDim.x + threadIdx.x), (int)(gridDim.y * blockDim.x));
  }
}

// Micro-tile level for the listed unit pairs.  The grid strides over the list in x; the gridDim.y blocks of
// one x share the micro-tile pairs of an entry, so that a pair of large groups (millions of micro-tile pairs
// in one entry) does not hang on a single block.
template <bool LIST>
__global__ __launch_bounds__(256) void k_bound_refine(const BoundL2Args fine, const UnitTable ut, const BoundPairs bp) {
  const unsigned long long n = *bp.count < bp.cap ? *bp.count : bp.cap;
  for (unsigned long long e = blockIdx.x; e < n; e += gridDim.x) {
    const unsigned long long v = bp.list[e];
    refine_unit_pair<LIST>(fine, ut, (int)(v >> 48), (int)((v >> 24) & 0xffffffull), (int)(v & 0xffffffull),
                     (int)(blockIdx.y * blockDim.x + threadIdx.x), (int)(gridDim.y * blockDim.x));
  }
}

// Tile lists from the bitmap.  A wave takes kBitmapRowsPerLane x 64 (relation, head tile) rows: every lane counts
// the surviving tail tiles of its rows (almost all rows are empty); the wave reserves its part of the column list and
// of the active-row list with ONE atomic each (thousands of atomics on the same two counters cost more than the
// whole scan), and the rows that have tiles are then written out by the whole wave, one row after the other, tile
// numbers ascending.
constexpr int kBitmapRowsPerLane = 8;
constexpr int kBitmapShortWords = 64;
__host__ __device__ inline int bitmap_rows_per_lane(int words_per_row) { return words_per_row <= kBitmapShortWords ? kBitmapRowsPerLane : 1; }
__global__ __launch_bounds__(256) void k_rows_from_bitmap(const uint32_t* __restrict__ bitmap, int words_per_row,
                                                         int64_t n_rows, uint32_t* __restrict__ row_start,
                                                         uint32_t* __restrict__ row_count, uint32_t* __restrict__ cols,
                                                         unsigned long long* __restrict__ total,
                                                         uint32_t* __restrict__ active_rows,
                                                         unsigned int* __restrict__ n_active,
                                                         uint32_t* __restrict__ tile_rows,        // may be NULL: the row of every entry of cols
                                                         int nH = 1, int h0 = 0, int h1 = 0x7fffffff,     // window: only head tiles [h0, h1)
                                                         int t0 = 0, int t1 = 0x7fffffff,                 // ... and tail tiles [t0, t1) count
                                                         const unsigned int* skip = nullptr,              // non-zero: the lists exist already, nothing to do
                                                         unsigned long long* tiles_total = nullptr) {     // running total of listed tiles (with skip)
  if (skip && *skip) return;
  // word i of a row holds tail tiles 32 i .. 32 i + 31: the bits of those inside [t0, t1)
  auto col_mask = [=](int i) -> uint32_t {
    const int lo = t0 - 32 * i, hi = t1 - 32 * i;
    if (hi <= 0 || lo >= 32) return 0u;
    const uint32_t mlo = lo <= 0 ? 0xffffffffu : 0xffffffffu << lo;
    const uint32_t mhi = hi >= 32 ? 0xffffffffu : (1u << hi) - 1u;
    return mlo & mhi;
  };
  auto row_in = [=](int64_t row) -> bool { const int tH = (int)(row % nH); return tH >= h0 && tH < h1; };
  const int lane = threadIdx.x & 63;
  // rows of up to kBitmapShortWords words are counted one per lane, kBitmapRowsPerLane of them; longer rows by the
  // whole wave, one after the other, 64 per wave
  const int rpl = bitmap_rows_per_lane(words_per_row);
  const int64_t row0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * (64 * rpl);
  if (row0 >= n_rows) return;                                  // whole waves leave together
  uint32_t cnt[kBitmapRowsPerLane];
#pragma unroll
  for (int k = 0; k < kBitmapRowsPerLane; ++k) {
    const int64_t base_row = row0 + k * 64;
    cnt[k] = 0;
    if (k >= rpl) continue;
    if (words_per_row <= kBitmapShortWords) {   // short rows: every lane counts its own
      if (base_row + lane < n_rows && row_in(base_row + lane)) {
        const uint32_t* w = bitmap + (base_row + lane) * words_per_row;
        for (int i = 0; i < words_per_row; ++i) cnt[k] += __builtin_popcount(w[i] & col_mask(i));
      }
    } else {                                 // long rows: the wave counts them one after the other, words over lanes
      for (int rr = 0; rr < 64 && base_row + rr < n_rows; ++rr) {
        const uint32_t* w = bitmap + (base_row + rr) * words_per_row;
        uint32_t c = 0;
        for (int i = lane; i < words_per_row; i += 64) c += __builtin_popcount(w[i] & col_mask(i));
        for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
        if (lane == rr && row_in(base_row + rr)) cnt[k] = c;
      }
    }
  }
  // this lane's tiles and rows, their exclusive prefix over the wave, one reservation per wave
  uint32_t ltiles = 0, lrows = 0;
#pragma unroll
  for (int k = 0; k < kBitmapRowsPerLane; ++k) { ltiles += cnt[k]; lrows += cnt[k] ? 1u : 0u; }
  uint32_t ptiles = ltiles, prows = lrows;
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t ot = __shfl_up(ptiles, off, 64), orw = __shfl_up(prows, off, 64);
    if (lane >= off) { ptiles += ot; prows += orw; }
  }
  const uint32_t wtiles = __shfl(ptiles, 63, 64), wrows = __shfl(prows, 63, 64);
  unsigned long long wbase = 0;
  unsigned int abase = 0;
  if (lane == 0 && wrows) {
    wbase = atomicAdd(total, (unsigned long long)wtiles);
    abase = atomicAdd(n_active, wrows);
    if (tiles_total) atomicAdd(tiles_total, (unsigned long long)wtiles);
  }
  wbase = ((unsigned long long)(uint32_t)__shfl((int)(uint32_t)(wbase >> 32), 0, 64) << 32) |
          (uint32_t)__shfl((int)(uint32_t)(wbase & 0xffffffffull), 0, 64);
  abase = (unsigned int)__shfl((int)abase, 0, 64);
  unsigned long long my_base = wbase + (ptiles - ltiles);
  unsigned int my_act = abase + (prows - lrows);
  unsigned long long bases[kBitmapRowsPerLane];
#pragma unroll
  for (int k = 0; k < kBitmapRowsPerLane; ++k) {
    const int64_t my_row = row0 + k * 64 + lane;
    bases[k] = cnt[k] ? my_base : 0ull;
    if (k < rpl && my_row < n_rows) {
      row_start[my_row] = (uint32_t)bases[k];
      row_count[my_row] = cnt[k];
      if (cnt[k]) active_rows[my_act++] = (uint32_t)my_row;   // rows that still have work, in any order
    }
    my_base += cnt[k];
  }
  if (!wrows) return;
#pragma unroll 1
  for (int k = 0; k < rpl; ++k) {
    uint32_t c = 0;
    unsigned long long bk = 0;
#pragma unroll
    for (int q = 0; q < kBitmapRowsPerLane; ++q) { c = (q == k) ? cnt[q] : c; bk = (q == k) ? bases[q] : bk; }
    unsigned long long live = __builtin_amdgcn_ballot_w64(c != 0u);
    while (live) {
      const int src = (int)__builtin_ctzll(live);
      live &= live - 1ull;
      const unsigned long long base = ((unsigned long long)(uint32_t)__shfl((int)(uint32_t)(bk >> 32), src, 64) << 32) |
                                      (uint32_t)__shfl((int)(uint32_t)(bk & 0xffffffffull), src, 64);
      const uint32_t* w = bitmap + (row0 + k * 64 + src) * words_per_row;
      // ascending order: words in chunks of 64, prefix of popcounts across lanes
      uint32_t run = 0;
      for (int i0 = 0; i0 < words_per_row; i0 += 64) {
        const int i = i0 + lane;
        uint32_t word = i < words_per_row ? (w[i] & col_mask(i)) : 0u;
        const uint32_t pc = __builtin_popcount(word);
        uint32_t pre = pc;
        for (int off = 1; off < 64; off <<= 1) {
          const uint32_t o = __shfl_up(pre, off, 64);
          if (lane >= off) pre += o;
        }
        uint32_t pos = run + pre - pc;
        while (word) {
          const int bit = __builtin_ctz(word);
          word &= word - 1;
          if (tile_rows) tile_rows[base + pos] = (uint32_t)(row0 + k * 64 + src);
          cols[base + pos++] = (uint32_t)(i * 32 + bit);
        }
        run += __shfl(pre, 63, 64);
      }
    }
  }
}

}  // namespace kgc

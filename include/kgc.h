/*
 * kgc -- TransE knowledge-graph completion as a threshold similarity join, on one AMD MI355X (gfx950).
 *
 * Given entity embeddings E (N x d) and relation vectors Rv (R x d), the join returns every triple
 * (h, r, t) in E x R x E with
 *
 *        dist_3(h, r, t) = || E[h] + Rv[r] - E[t] ||_p  <=  delta,        p in {1, 2}.
 *
 * This is the completion problem of Definition 1 (Section 3.1) for the TransE distance, after the
 * transformation of Section 4.3: connector_1(h, r) = h + r, connector_2(t, r) = t,
 * dist(a, b) = ||a - b||_p.  The threshold is inclusive (Section 3.1 includes equality), self
 * pairs h == t are included and nothing is filtered against an existing graph.  The paper calls the
 * distance threshold epsilon; it is named delta here because the paper also uses epsilon for the score.
 *
 * C ABI, plain pointers and sizes.  Unless marked "host", a pointer is a DEVICE pointer owned by the
 * caller: the library reads E / Rv, writes out_triples, and never frees or reallocates them.
 * Scratch memory is owned by the handle and released by kgc_destroy.  All work of a handle is
 * enqueued on the HIP stream given at creation.  A handle must not be used from two threads at once.
 */
#ifndef KGC_H
#define KGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kgc_handle kgc_handle;          /* opaque */

/* One result record (16 bytes).  h, r, t are 0-based row numbers in the caller's E / Rv (any
 * internal reordering is undone).  dist is the norm itself (not its square), rounded to float from
 * the double-precision value the hit decision was taken on. */
typedef struct { int32_t h, r, t; float dist; } kgc_triple;

/* storage type of E and Rv */
#define KGC_F32  0      /* IEEE float32 */
#define KGC_BF16 1      /* bfloat16 (upper 16 bits of a float32) */

/* pruning */
#define KGC_PRUNE_AUTO 0   /* = KGC_PRUNE_ON */
#define KGC_PRUNE_OFF  1   /* dense: every tile pair goes through the join kernel (Section 5.1's naive mode) */
#define KGC_PRUNE_ON   2   /* tile pairs are skipped when the pivot bound of Lemma 1 (Section 4.4) exceeds delta */

/* return codes */
#define KGC_OK            0
#define KGC_OVERFLOW      1    /* more hits than cap: *count is the true total, out_triples holds cap of them */
#define KGC_E_INVALID    -1    /* bad argument; nothing was launched */
#define KGC_E_NOMEM      -2    /* device or host allocation failed */
#define KGC_E_HIP        -3    /* a HIP call failed; see kgc_last_error */

/* Configuration of a handle.  A zero-filled struct selects the defaults. */
typedef struct {
    int32_t dtype;            /* KGC_F32 (default) or KGC_BF16: element type of E and Rv */
    int32_t max_d;            /* largest d this handle accepts; 0 = 960 (the compiled limit) */
    int32_t prune;            /* KGC_PRUNE_* */
    int32_t tile_cfg;         /* 0 = automatic choice of the L2 join kernel; > 0 forces a variant (for measurements):
                                 1-5   one block per tile pair, 128/256-row tiles (dense mode only)
                                 6-10  streaming: a block walks tail tiles, head and tail slices through LDS (any d)
                                 11-14 head tile resident in LDS, tail slices through LDS (d <= 250; 14, two 128 x 128
                                       blocks per CU, is the pruned default below 262,144 entities)
                                 15-18 head tile resident, tail fragments straight to registers, no barrier in the
                                       loop (15-16: d <= 282; 17: d <= 602; 18: d <= 282, one straight-line
                                       instantiation per number of K steps, the dense default).  Dense mode, and 15
                                       also pruned, walking tile lists: the pruned default from 262,144 entities on
                                 A variant that cannot run the request (pruned mode, d) fails with KGC_E_INVALID. */
    int64_t workspace_bytes;  /* cap on scratch held for staged operands; 0 = 16 GiB.  Larger joins run in relation batches */
    void*   stream;           /* hipStream_t to enqueue on; NULL = the default stream */
    float   group_radius;     /* pruning only: radius of entity groups as a multiple of delta; 0 = 2.0 */
    int32_t range_kib;        /* dense L2 join: KiB of staged tail rows one block walks (L2 blocking); 0 = automatic */
    int32_t factorised;       /* 1: dense L2 joins with d <= 282 use the relation-factorised kernel (one MFMA tile
                                 ||h - t||^2 per tile pair, then vector arithmetic per relation); same result set */
    int32_t reserved[3];      /* must be zero */
} kgc_config;

/* Counters and timings of the last kgc_join on a handle. */
typedef struct {
    uint64_t triples_total;     /* N * N * R */
    uint64_t tiles_total;       /* tile triples (r, head tile, tail tile) of the dense problem */
    uint64_t tiles_evaluated;   /* tile triples that went through the join kernel */
    uint64_t tiles_pruned;      /* tiles_total - tiles_evaluated */
    uint64_t pairs_evaluated;   /* (h, r, t) scored by the join kernel: N * N * R with pruning off; with pruning on,
                                   tiles_evaluated * tile_m * tile_n (padding rows of the grouped layout included) */
    uint64_t candidates;        /* triples that passed the low-precision stage and were re-scored in double */
    uint64_t emitted;           /* hits found (= *count) */
    uint64_t join_launches;     /* launches of the join kernel */
    uint64_t groups;            /* entity groups formed for pruning (0 when pruning is off) */
    float    ms_total;          /* whole call on the stream, from HIP events */
    float    ms_precompute;     /* norm / operand staging kernels (a1) */
    float    ms_prune;          /* grouping + tile bound kernels (a2) */
    float    ms_join;           /* join kernel launches only (a3 or a4, with the compaction a5 inside) */
    int32_t  tile_m, tile_n;    /* tile shape used (heads x tails) */
    int32_t  k_padded;          /* contraction length after appending the norm columns and padding (L2) */
    int32_t  relation_batches;
    int32_t  join_variant;      /* which join kernel ran: 0 = L1 (VALU); for L2 the tile_cfg number that was used,
                                   100 = the relation-factorised kernel */
    int32_t  exact_blocks;      /* 32 x 32 blocks of pairs that the pruned L2 joins re-scored as whole blocks in double
                                   precision (their candidates come in patches); 0 for the other paths */
} kgc_stats;

/* Create a handle.  cfg may be NULL (defaults).  Returns KGC_OK and stores the handle in *out (host),
 * or a negative code and stores NULL. */
int kgc_create(const kgc_config* cfg, kgc_handle** out);

/* The join (Definition 1, Section 3.1; distance of Section 4.3).
 *   E           N x d row-major, contiguous, of the handle's dtype           (device)
 *   Rvecs       R x d row-major, contiguous, same dtype                      (device)
 *   p           1 or 2
 *   delta       threshold on the norm; negative => empty result
 *   out_triples room for cap records, 16-byte aligned                        (device; may be NULL iff cap == 0)
 *   count       receives the number of qualifying triples, which may exceed cap (host)
 * On KGC_OK the first *count records are the result, in unspecified order, each triple once.
 * On KGC_OVERFLOW the buffer holds an arbitrary cap-subset of the result and *count is the true total.
 * N == 0 or R == 0 is valid and yields *count == 0.  Non-finite values in E, Rvecs: undefined result.
 * KGC_E_INVALID: p not in {1,2}; d < 1 or d > max_d; N > 2^31 - 64 or R > 2^31 - 1; delta NaN;
 * a NULL pointer where data is required.  The call synchronises the stream once, to read the count.
 *
 * How the set is found: the L2 join scores tile pairs with a bf16 MFMA contraction whose result is a
 * conservative filter; the L1 join uses float32 vector arithmetic as the filter.  Every triple that
 * passes the filter is re-scored from the caller's E / Rv in double precision in the order
 * (E[h] + Rv[r]) - E[t], dimensions summed by a wave-level tree, and the <= delta decision is taken
 * on that double value. */
int kgc_join(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R,
             int32_t p, float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count);

/* Kernel 1 on its own, for testing: squared L2 norms the pivot bound and the contraction use.
 *   nB[t]        = || bf16(E[t]) ||^2                 N floats      (device)
 *   nA[r*N + h]  = || bf16(E[h] + Rv[r]) ||^2         R*N floats    (device)
 * With the zero vector as pivot (Section 4.5) these are the squares of distB and distA, taken on the
 * bf16-rounded operands the contraction sees.  Either output may be NULL. */
int kgc_norms(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R,
              float* nB, float* nA);

/* The same join restricted to the relations r_begin <= r < r_end (0 <= r_begin <= r_end <= R); r in the
 * records is still the row number in Rvecs.  The join over [0, R) is the disjoint union of the joins over
 * any partition of [0, R) into ranges, which lets a caller bound the output of one call (a range whose
 * result overflows cap can be split and run again) and drain a result larger than its buffer range by
 * range -- the relation-wise form of the partition-based join of Section 4.7.  kgc_join is this call with
 * the range [0, R).  An empty range yields *count == 0. */
int kgc_join_range(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                   float delta, int32_t r_begin, int32_t r_end, kgc_triple* out_triples, uint64_t cap, uint64_t* count);

/* kgc_join for callers that cannot allocate device memory while they run: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same dense join (every tile pair goes through the join kernel, the
 * handle's pruning setting is ignored; same kernels, result set, output, count, overflow and error conventions as
 * kgc_join), but ALL of its scratch -- counters, filter threshold, slot order, staged operands and norms -- lies
 * in one 48 MiB array that is part of the library's device code; the call allocates and frees nothing (no hipMalloc,
 * hipFree, event creation or host allocation; the array's address on the handle's device was looked up by
 * kgc_create).  Relations run in batches of as many staged head operands as fit the array.
 * KGC_E_INVALID when the fixed part alone does not fit (it needs about (N + 255) * (64 * ceil((d + 6) / 32) + 4) * 2
 * bytes for p = 2: e.g. N <= 87,000 at d = 100, N <= 50,000 at d = 200), when the handle was created with
 * factorised = 1, or when the handle's device is not the current device.  Every GPU holds ONE such array, shared by
 * every handle and call on that GPU: calls that overlap in time on one GPU race on it and must be serialised by the
 * caller; a call leaves its operands behind, and the next call overwrites what it uses.  Per-batch kernel times
 * are not taken: stats.ms_join spans operand staging and join launches together. */
int kgc_join_static(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                    float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count);

/* The join in its general form (Section 4.3): for a model that can be transformed to a metric space the
 * caller supplies the connector outputs and the library joins them under dist(a, b) = ||a - b||_p:
 *   A   R x N x d   a_{r,h} = connector_1(h, r), row-major, contiguous, of the handle's dtype          (device)
 *   B   N x d when b_per_relation == 0 (connector_2 does not depend on r; TransE: b = t), else R x N x d
 *       with b_{r,t} = connector_2(t, r)                                                               (device)
 * finds every (h, r, t) with ||A[r][h] - B[r or 0][t]||_p <= delta.  TransE is A[r][h] = E[h] + Rv[r], B = E; the
 * structured-embedding model of the same section is A[r] = E W1_r^T, B[r] = E W2_r^T with p = 1.  Output, count,
 * overflow and error conventions are those of kgc_join; the exact stage scores (double)a - (double)b.  The
 * relations run through the join kernels of kgc_join in batches.  With pruning on (the handle's setting) the
 * rows of B (of its first relation) are grouped, every A[r] and B[r] is summarised in that order, and tile pairs
 * whose pivot bound (Lemma 1, Section 4.4) exceeds delta are skipped; the result does not depend on it. */
int kgc_join_ab(kgc_handle* hd, const void* A, const void* B, int64_t N, int32_t d, int32_t R, int32_t b_per_relation,
                int32_t p, float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count);

/* Where a join over blocks stands.  Zero it before the first call of a join; the library updates it. */
typedef struct {
    uint64_t unit;        /* units (relation range, head block, tail block) done so far: the next call starts with this one */
    uint64_t units;       /* units of the whole join (known after the first call) */
    uint64_t need;        /* after KGC_OVERFLOW: the number of triples of the unit that did not fit */
    uint64_t reserved;
} kgc_cursor;

/* The partition-based join (Section 4.7): kgc_join cut into units that are joined one after the other, with a
 * cursor, so that a result larger than the output buffer can be drained piece by piece.
 *   block_rows   rows per block of the join's row order (rounded up to a multiple of 256).  With pruning on that order
 *                is the grouped one (similar entities are neighbours), as the section cuts its sorted arrays; without
 *                pruning it is the entity order
 *   rel_block    relations per unit
 *   cursor       host; all zero to start a join.  Units run in the order (relation range, head block, tail block)
 * Each call runs units from cursor->unit on and appends their triples to out_triples until all are done (KGC_OK,
 * cursor->unit == cursor->units) or the next unit's triples do not fit what is left of the buffer (KGC_OVERFLOW:
 * *count triples of COMPLETE units are in the buffer, cursor->unit names the unit that is still to be done and
 * cursor->need its size; the caller takes the triples away and calls again with the same arguments and cursor).  A
 * unit larger than the whole buffer returns KGC_OVERFLOW with *count == 0: call again with cap >= cursor->need, or
 * start over with smaller blocks.  No triple is returned twice, and the union over the calls is the result of kgc_join.
 * The handle keeps the row order, the summaries and the staged tail operands of the join between the units and the
 * calls (and the bound test of a relation range between that range's units); any other call on the handle except
 * kgc_get_stats / kgc_last_error discards them, after which a continued pruned join is refused (KGC_E_INVALID): its
 * grouped order cannot be made again identically.  They are made anew when the cursor is zero or E, Rvecs, N, d, p or
 * delta differ; the caller must not change the contents of E or Rvecs between the calls of one join.
 * Other conventions (dtype, layout, errors) as kgc_join; the relation-factorised form is not available here. */
int kgc_join_blocks(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                    float delta, int64_t block_rows, int32_t rel_block, kgc_cursor* cursor, kgc_triple* out_triples,
                    uint64_t cap, uint64_t* count);

/* The structured-embedding instance of the general form (Section 4.3): connector_1(h, r) = W_lhs[r] h and
 * connector_2(t, r) = W_rhs[r] t, joined under ||a - b||_p (the model's own norm is p = 1; p = 2 is accepted).
 *   E       N x d row-major, contiguous, of the handle's dtype                                       (device)
 *   W_lhs   R x d x d, W_lhs[r][i][j] row-major (a_i = sum_j W_lhs[r][i][j] h_j), same dtype        (device)
 *   W_rhs   R x d x d, the same for the tail side                                                    (device)
 * The library forms the connector rows itself, relation batch by relation batch, in float32 (products of the
 * stored values, float32 accumulation) in buffers of the handle: 2 * batch * N * d * 4 bytes, a batch being as many
 * relations as fit a quarter of config.workspace_bytes (at most 4 GiB a side); the caller never holds R x N x d.
 * Each batch then runs through the kernels of kgc_join_ab on those rows, and the exact stage scores the stored
 * float32 connector rows in double.  A connector element therefore carries a rounding error of about
 * sqrt(d) * 2^-24 of |W row| |e|, a distance one of about sqrt(2 d) (p = 2) or 2 d (p = 1) times that: triples whose
 * exact distance lies that close to delta may fall on either side.  Output, count, overflow and error conventions are
 * those of kgc_join; kgc_get_stats reports the sums over the batches. */
int kgc_join_se(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* W_lhs, const void* W_rhs, int32_t R,
                int32_t p, float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count);

/* The top-1 score of Section 3.3: the triple with the smallest dist_3(h, r, t) over E x R x E, or, with
 * exclude_self != 0, over the triples with h != t (the second quantity that section looks at).
 *   out   receives the triple and its distance (host).  h = r = t = -1 and dist = +inf when no triple is
 *         eligible (N == 0, R == 0, or exclude_self with N == 1): that is KGC_OK, not an error.
 * Same E / Rvecs / p conventions and error codes as kgc_join.  Found by joins with a shrinking threshold,
 * starting from the smallest of 65,536 sampled triples; the handle's pruning setting applies.  Among triples
 * whose distances agree to float precision the smallest (r, h, t) is returned.  Synchronises the stream a
 * few times. */
int kgc_top1(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
             int32_t exclude_self, kgc_triple* out);

/* The k triples with the smallest distances: the top-k scores the experiments of Section 3.3 rank by (kgc_top1 is
 * k = 1; k up to 65536), optionally without self pairs.
 *   out_triples  room for k records, 16-byte aligned, in no particular order                 (device)
 *   found        receives min(k, number of eligible triples)                                 (host)
 * Joins with a growing threshold, started just above the top-1 bound of kgc_top1, until one returns at least
 * k records; those are cut to the k smallest by a radix select on the distance (among records whose distances
 * agree to float precision with the k-th, which ones are returned is unspecified). */
int kgc_topk(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
             int32_t exclude_self, uint64_t k, kgc_triple* out_triples, uint64_t* found);

/* kgc_topk over the relations r_begin <= r < r_end only (kgc_topk is the range [0, R)); with a range of one
 * relation, the k best (h, t) pairs of that relation: the per-relation ranking of Section 3.3. */
int kgc_topk_range(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                   int32_t exclude_self, int32_t r_begin, int32_t r_end, uint64_t k, kgc_triple* out_triples,
                   uint64_t* found);

/* Copy the statistics of the last kgc_join into *out (host). */
int kgc_get_stats(const kgc_handle* hd, kgc_stats* out);

/* Message of the last failure on this handle ("" if none).  The string lives as long as the handle. */
const char* kgc_last_error(const kgc_handle* hd);

/* Release the handle and its scratch memory.  NULL is allowed. */
void kgc_destroy(kgc_handle* hd);

/* Calibration of the roofline of the L2 join (measurement support, Section 5's question of what the hardware
 * sustains): a loop of nothing but bf16 32x32x16 MFMAs on a wave tile of the join's kind, on pseudo-random operands,
 * run for about ms_target milliseconds so that the clock the chip settles on under that load is the one measured.
 *   wave_tile  0: 4 x 2 accumulator blocks (128 x 64, two waves per SIMD, the join kernels' shape); 1: 4 x 4 (one wave per SIMD)
 *   feed       0: operands stay in registers; 1: head fragments read from LDS every K step, as in the join;
 *              2: ... and tail fragments read from global memory through the vector cache in the join's pattern
 *   stream     hipStream_t to run on (NULL = default stream)
 *   tflops     receives the sustained rate in TFLOP/s (host);  ms receives the duration of the timed launch (host)
 * Allocates and frees its own scratch.  KGC_E_INVALID on a bad argument. */
int kgc_calibrate_mfma(int32_t wave_tile, int32_t feed, int32_t ms_target, void* stream, double* tflops, float* ms);

/* Library version, "major.minor.patch". */
const char* kgc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KGC_H */

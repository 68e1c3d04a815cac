// Host side of the kgc C ABI (see include/kgc.h): argument checks, scratch management, launch order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kgc_kernels.h"
#include "kgc_dense.h"
#include "kgc_calibrate.h"
#include "kgc_prune.h"

using namespace kgc;

// Scratch of kgc_join_static (the entry point for callers that cannot allocate): one array per GPU, held from the
// moment the code object is loaded until the process ends.  In host code this name is only a stand-in for the
// symbol; the array's device address is taken once per device with hipGetSymbolAddress (static_scratch_ptr).
constexpr size_t kStaticScratchBytes = 48u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxD = 960;                      // keeps kernel 1's LDS tile under 64 KiB
constexpr int64_t kFewEntities = 32768;        // grouping: up to here three covering rounds instead of six
constexpr int64_t kSlotAlign = 256;            // rows are padded to a multiple of the largest tile
constexpr int64_t kDefaultWorkspace = 16ll << 30;
constexpr size_t kBoundPairCap = 8u << 20;      // surviving (relation, unit, unit) entries of one batch kept in the list
constexpr int64_t kL2RangeBytes = 1ll << 20;
constexpr int64_t kL2RangeBytesResident = 4ll << 20;   // head-resident blocks leave the whole L2 to the tail rows
constexpr int64_t kL2RangeBytesSplit = 3ll << 20;      // ... and a B that has to be cut anyway is cut finer

// Bytes of staged tail rows per launch range of a head-resident kernel.  A B that fits the L2 is one range; a larger
// one is cut into 3 MiB ranges: measured on the d = 200 workload they cost the same time as 4 MiB ranges and miss
// the L2 for 136 GB per launch instead of 237 GB.
static inline int64_t resident_range_bytes(int64_t tail_bytes) {
  return tail_bytes <= kL2RangeBytesResident ? kL2RangeBytesResident : kL2RangeBytesSplit;
}
constexpr size_t kMaxLds = 160 * 1024;         // LDS per workgroup on gfx950
constexpr int64_t kMaxTileList = 1ll << 30;    // entries of the surviving-tile list per relation batch (4 bytes each)
constexpr unsigned int kExactListCap = 1u << 20;   // accumulator blocks one batch may list for the exact stage (16 bytes each)

struct DevBuf {
  void* p = nullptr;
  size_t bytes = 0;
};

}  // namespace

struct kgc_handle {
  kgc_config cfg{};
  hipStream_t stream = nullptr;
  int device = 0;
  std::string err;
  kgc_stats stats{};
  DevBuf slot_ent, opB, opA, normsB, normsA, counters, params;
  // pruning scratch
  DevBuf gstate, unc_a, unc_b, group_of, piv_ent, best, gsize, goff, gfill, cent, rad, bitmap, row_start, row_count, cols, tile_rows;
  DevBuf active_rows, cnorm, gram, relu, reln, asg_a, asg_b, limr;
  // every DevBuf member must also be listed in kgc_destroy
  DevBuf top1_buf, top1_state;                 // top-1 search: records of the inner joins, Top1State
  DevBuf unit_first, unit_n, cent_u, rad_u, cnorm_u, gram_u, relu_u, pair_list, pair_count;   // two-level bound test
  // what the handle's grouping, summaries and staged tail operands were made for (kgc_join_blocks reuses them)
  struct Prep {
    bool valid = false;
    const void* E = nullptr; const void* Rv = nullptr;
    int64_t N = 0; int d = 0, p = 0, dtype = 0, prune = 0, tile_id = 0; float delta = 0.f, group_radius = 0.f;
    int64_t Nslots = 0; uint64_t n_groups = 0; UnitTable ut{};
    bool bitmap_valid = false; int64_t bm_r0 = 0, bm_r1 = 0;     // the bitmap holds the bound test of these relations
  } prep;
  DevBuf se_a, se_b;                           // connector rows of a relation batch (kgc_join_se)
  DevBuf xlist;                                // accumulator blocks listed for the exact stage (L2 joins)
  unsigned int xcap = kExactListCap;           // its length in entries: grows when a batch wanted to list more
  int list_seg_cap = 0;                        // > 0: the pruned barrier-free kernel keeps at most this many entries of a row's tile list in the LDS (tests)
  unsigned pairs_grid = 512;                   // workgroups of the tile-at-a-time kernel: two per compute unit (tests set fewer, so that a workgroup walks several batches of tiles)
  DevBuf zero_row, cent_a, rad_a;              // kgc_join_ab: the zero relation row; micro-tile summaries of A[r]
  DevBuf top1_a, top1_b, top1_pick, top_samples, topk_state;            // ... and the operands / entity samples of its sub-sampled dense pass
  int no_self = 0;                             // set by kgc_top1 around its inner joins: drop h == t
  bool static_mode = false;                    // inside kgc_join_static: the DevBufs point into the static array, nothing may allocate
  int64_t ws_override = 0;                     // ... and the staged operands of a relation batch get this many bytes
  GroupState* host_gstate = nullptr;           // pinned
  DevCounters* host_counters = nullptr;        // pinned
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  std::vector<hipEvent_t> join_ev;             // pairs around each join launch
};

namespace {

int fail(kgc_handle* h, int code, const char* what, hipError_t e = hipSuccess) {
  if (h) {
    h->err = what;
    if (e != hipSuccess) {
      h->err += ": ";
      h->err += hipGetErrorString(e);
    }
  }
  return code;
}

#define KGC_HIP(h, call)                                                        \
  do {                                                                          \
    hipError_t _e = (call);                                                     \
    if (_e != hipSuccess)                                                       \
      return fail((h), _e == hipErrorOutOfMemory ? KGC_E_NOMEM : KGC_E_HIP, #call, _e); \
  } while (0)

int ensure(kgc_handle* h, DevBuf& b, size_t bytes) {
  if (b.bytes >= bytes && b.p) return KGC_OK;
  if (h->static_mode) return fail(h, KGC_E_INVALID, "kgc_join_static: a buffer was not laid out in the static scratch");
  if (b.p) {
    KGC_HIP(h, hipFree(b.p));
    b.p = nullptr;
    b.bytes = 0;
  }
  if (bytes == 0) bytes = 256;
  KGC_HIP(h, hipMalloc(&b.p, bytes));
  b.bytes = bytes;
  return KGC_OK;
}

void release(DevBuf& b) {
  if (b.p) (void)hipFree(b.p);
  b.p = nullptr;
  b.bytes = 0;
}

// Device address of the static scratch array on `device` (which must be the current device): every GPU holds its own
// copy of the array at its own address, looked up once and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch_ptr(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return KGC_E_INVALID;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KGC_E_HIP;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return KGC_OK;
}

struct TileCfg {
  int bm, bn, threads;
  void (*tile_kernel)(const JoinArgs);            // one block per tile pair
  void (*stream_kernel)(const JoinStreamArgs);    // one block per (relation, head tile), streaming over tail tiles
  void (*listed_kernel)(const JoinStreamArgs);    // the same kernel walking the tile lists of pruned mode
  bool head_resident;                             // stream_kernel keeps the head tile's K slices in LDS (dynamic LDS)
  size_t static_lds;                              // head-resident kernels: bytes of static LDS beside the tiles (none today)
  int blocks_per_cu;                              // head-resident kernels: workgroups meant to share one CU's LDS
  int tail_buffers;                               // head-resident kernels: tail slices held in LDS (0: tail rows bypass LDS)
};

// Tile variants of kernel 2 (tile_cfg = index + 1).
const TileCfg kL2Tiles[] = {
    {128, 128, 256, k_join_l2<128, 128, 2, 2>, nullptr, nullptr, false, 0, 1, 2},
    {256, 128, 256, k_join_l2<256, 128, 2, 2>, nullptr, nullptr, false, 0, 1, 2},
    {256, 256, 256, k_join_l2<256, 256, 2, 2>, nullptr, nullptr, false, 0, 1, 2},
    {128, 128, 512, k_join_l2<128, 128, 4, 2>, nullptr, nullptr, false, 0, 1, 2},
    {256, 256, 512, k_join_l2<256, 256, 4, 2>, nullptr, nullptr, false, 0, 1, 2},
    {256, 256, 256, nullptr, k_join_l2_stream<256, 256, 2, 2, 1, false>, k_join_l2_stream<256, 256, 2, 2, 1, true>, false, 0, 1, 2},
    {256, 128, 256, nullptr, k_join_l2_stream<256, 128, 2, 2, 2, false>, k_join_l2_stream<256, 128, 2, 2, 2, true>, false, 0, 1, 2},
    {128, 128, 256, nullptr, k_join_l2_stream<128, 128, 2, 2, 2, false>, k_join_l2_stream<128, 128, 2, 2, 2, true>, false, 0, 1, 2},
    {256, 256, 512, nullptr, k_join_l2_stream<256, 256, 4, 2, 1, false>, k_join_l2_stream<256, 256, 4, 2, 1, true>, false, 0, 1, 2},
    {128, 256, 256, nullptr, k_join_l2_stream<128, 256, 2, 2, 2, false>, k_join_l2_stream<128, 256, 2, 2, 2, true>, false, 0, 1, 2},
    {256, 256, 512, nullptr, k_join_l2_ares<256, 256, 4, 2, 1, 512, false>, k_join_l2_ares<256, 256, 4, 2, 1, 512, true>, true, 0, 1, 2},
    {256, 256, 512, nullptr, k_join_l2_ares<256, 256, 2, 4, 1, 512, false>, k_join_l2_ares<256, 256, 2, 4, 1, 512, true>, true, 0, 1, 2},
    {256, 128, 512, nullptr, k_join_l2_ares<256, 128, 4, 2, 1, 512, false>, k_join_l2_ares<256, 128, 4, 2, 1, 512, true>, true, 0, 1, 2},
    {128, 128, 256, nullptr, k_join_l2_ares<128, 128, 2, 2, 2, 256, false>, k_join_l2_ares<128, 128, 2, 2, 2, 256, true>, true, 0, 2, 2},
    {256, 256, 512, nullptr, k_join_l2_direct<256, 2, 4, kEpiJoin>, k_join_l2_direct<256, 2, 4, kEpiJoin, true>, true, 0, 1, 0},
    {256, 256, 512, nullptr, k_join_l2_direct<256, 1, 8, kEpiJoin>, nullptr, true, 0, 1, 0},
    {128, 256, 512, nullptr, k_join_l2_direct<128, 1, 8, kEpiJoin>, nullptr, true, 0, 1, 0},
    {256, 256, 512, nullptr, k_join_l2_dense<1>, nullptr, true, 0, 1, 0},      // placeholder: see dense_kernel_for
};
constexpr int kDefaultL2Tile = 8;                 // index into kL2Tiles: streaming, 256 x 256, 8 waves
constexpr int kResidentL2Tile = 13;               // head-resident, 128 x 128, 4 waves, two blocks per CU (pruned default)
constexpr int kResidentLargeL2Tile = 11;          // head-resident, 256 x 256, 8 waves (2 x 4): pruned joins over many entities
constexpr int64_t kResidentLargeN = 1 << 18;      // ... from this many on: rows then hold many surviving tiles each, and the
                                                  // larger wave tile (half the LDS reads per MFMA) pays; below, the finer
                                                  // tiles follow the surviving patches more closely and balance better
// the pruned default for N entities and KS slices (both head-resident shapes need KS <= 8 to fit their LDS)
constexpr int kDirectL2Tile = 14;                 // head-resident and barrier-free, 8 waves (2 x 4): dense joins, and pruned joins over many entities
inline int pruned_l2_tile(int64_t N, int KS, int fallback) {
  if (((size_t)KS * 128 + 2 * 128) * kSliceK * 2 * 2 > kMaxLds) return fallback;
  if (N < kResidentLargeN) return kResidentL2Tile;
  // many entities: the barrier-free form walking the row's tile list, which sits in the LDS behind the head slices
  // (measured on the 10^6-entity workload: 610 ms of join per step against 647 ms)
  if ((size_t)KS * 256 * kSliceK * 2 + 16384 <= kMaxLds) return kDirectL2Tile;      // (room for 4,096 tiles of a row's list at a time)
  return kResidentLargeL2Tile;
}
constexpr int kDenseL2Tile = 17;                  // the same with a straight-line tile body per number of K steps (dense default)
constexpr int kDirectMaxKS = 9;                   // its head tile then takes 144 of the 160 KiB of LDS
constexpr int kDirectHalfL2Tile = 16;             // the same with a 128-row head tile (wave tile 128 x 32), for larger d
constexpr int kDirectHalfMaxKS = 19;              // 152 KiB
constexpr int kNumL2Tiles = (int)(sizeof(kL2Tiles) / sizeof(kL2Tiles[0]));

int check_common(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R) {
  if (!hd) return KGC_E_INVALID;
  const int max_d = hd->cfg.max_d > 0 ? std::min(hd->cfg.max_d, kMaxD) : kMaxD;
  if (d < 1 || d > max_d) return fail(hd, KGC_E_INVALID, "d must be in [1, max_d]");
  if (N < 0 || N > (int64_t)2147483647 - 64) return fail(hd, KGC_E_INVALID, "N out of range");
  if (R < 0) return fail(hd, KGC_E_INVALID, "R out of range");
  if (N > 0 && !E) return fail(hd, KGC_E_INVALID, "E is NULL");
  if (R > 0 && !Rvecs) return fail(hd, KGC_E_INVALID, "Rvecs is NULL");
  const uintptr_t al = hd->cfg.dtype == KGC_BF16 ? 2 : 4;
  if (((uintptr_t)E % al) || ((uintptr_t)Rvecs % al)) return fail(hd, KGC_E_INVALID, "E / Rvecs misaligned");
  return KGC_OK;
}

// Which vector reads the exact stage may use on the caller's arrays: decided here, from the addresses, d and the
// strides (multiples of d), and handed to the kernels in the context.
void set_alignment(RecheckCtx& cx) {
  auto al = [](const void* p, uintptr_t a) { return ((uintptr_t)p % a) == 0; };
  cx.base16 = al(cx.E, 16) && al(cx.Et, 16) && al(cx.Rv, 16) ? 1 : 0;
  const uintptr_t four = cx.dtype == KGC_BF16 ? 8 : 16;
  cx.vec_ok = (cx.d % 4 == 0 && al(cx.E, four) && al(cx.Et, four) && al(cx.Rv, four)) ? 1 : 0;
}

int group_rows(kgc_handle* hd, const void* E, int64_t N, int32_t d, int32_t p, float delta, int KS, int k16, int64_t* Nslots_out,
               uint64_t* n_groups_out, UnitTable* ut_out);        // further down

// the exact stage of the blocks a pruned L2 join kernel has listed (instantiated per storage type and row alignment)
void launch_exact_blocks(hipStream_t st, const ExactEntry* list, const unsigned int* count, unsigned int cap,
                         unsigned long long* total, unsigned int* need, const RecheckCtx& cx) {
  const bool bf = cx.dtype == KGC_BF16, vec = cx.vec_ok != 0;
  auto kern = bf ? (vec ? k_exact_blocks<true, true> : k_exact_blocks<true, false>)
                 : (vec ? k_exact_blocks<false, true> : k_exact_blocks<false, false>);
  hipLaunchKernelGGL(kern, dim3(256), dim3(kExactWaves * 64), 0, st, list, count, cap, total, need, cx);      // one workgroup per compute unit
}

// out[i][j] = x_i . y_j, one wave per 32 x 32 results on the float32 matrix pipes (k_small_dot): X rows of the storage
// type, Y rows float32
void launch_small_dot(hipStream_t st, const void* X, int dtype, int64_t n_rows, const float* Y, int64_t n_cols, int d, float* out) {
  const bool bf = dtype == KGC_BF16;
  const bool vec = d % 4 == 0 && (uintptr_t)X % (bf ? 8 : 16) == 0 && (uintptr_t)Y % 16 == 0;
  auto kern = bf ? (vec ? k_small_dot<true, true> : k_small_dot<true, false>)
                 : (vec ? k_small_dot<false, true> : k_small_dot<false, false>);
  hipLaunchKernelGGL(kern, dim3((unsigned)((n_cols + 31) / 32), (unsigned)((n_rows + 31) / 32), 1), dim3(64), 0, st,
                     X, n_rows, Y, n_cols, d, out);
}

// Blocks for `items` work items, `per_block` each.  A launch may hold fewer than 2^32 threads per grid dimension, so
// the count stops at 2^24 - 1 blocks (of at most 256 threads): enough for every per-row or per-slot kernel here
// (N < 2^31); kernels that can be asked for more (k_fill_u32, the staging kernels) stride over their items.
// Wait for an event that is usually a fraction of a millisecond away: polling it saves the wake-up of a blocking
// wait (tens of microseconds, twice per pruned join of half a millisecond); a join that takes longer falls back to
// the blocking wait and leaves the core alone.
hipError_t wait_event(hipEvent_t ev) {
  for (int i = 0; i < 4000; ++i) {
    const hipError_t q = hipEventQuery(ev);
    if (q != hipErrorNotReady) return q;
  }
  return hipEventSynchronize(ev);
}

int grid_for(int64_t items, int per_block) {
  return (int)std::min<int64_t>((items + per_block - 1) / per_block, (1 << 24) - 1);
}

}  // namespace

extern "C" {

const char* kgc_version(void) { return "0.1.0"; }

int kgc_create(const kgc_config* cfg, kgc_handle** out) {
  if (!out) return KGC_E_INVALID;
  *out = nullptr;
  kgc_config c{};
  if (cfg) c = *cfg;
  if (c.dtype != KGC_F32 && c.dtype != KGC_BF16) return KGC_E_INVALID;
  if (c.prune < KGC_PRUNE_AUTO || c.prune > KGC_PRUNE_ON) return KGC_E_INVALID;
  if (c.max_d < 0 || c.max_d > kMaxD || c.workspace_bytes < 0 || c.tile_cfg < 0 || c.tile_cfg > kNumL2Tiles)
    return KGC_E_INVALID;
  if (!(c.group_radius >= 0.f) || c.range_kib < 0 || c.factorised < 0 || c.factorised > 1) return KGC_E_INVALID;
  for (int v : c.reserved)
    if (v != 0) return KGC_E_INVALID;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return KGC_E_HIP;
  kgc_handle* h = new (std::nothrow) kgc_handle();
  if (!h) return KGC_E_NOMEM;
  h->cfg = c;
  h->stream = (hipStream_t)c.stream;
  if (hipGetDevice(&h->device) != hipSuccess) { delete h; return KGC_E_HIP; }
  {   // set-up for kgc_join_static: the address of this device's static scratch, so that the call itself looks nothing up
    void* sp = nullptr;
    const int src = static_scratch_ptr(h->device, &sp);
    if (src != KGC_OK) { delete h; return src; }
  }
  h->err.reserve(256);          // later error messages fit without a host allocation
  // the first length of the exact stage's block list (it grows by itself; tests set it small to see it grow)
  if (const char* e = std::getenv("KGC_EXACT_LIST_CAP")) h->xcap = (unsigned int)std::max(1L, std::atol(e));
  if (const char* e = std::getenv("KGC_TILE_LIST_SEGMENT")) h->list_seg_cap = (int)std::max(1L, std::atol(e));
  if (const char* e = std::getenv("KGC_PAIRS_GRID")) h->pairs_grid = (unsigned)std::min(512L, std::max(1L, std::atol(e)));
  if (hipHostMalloc((void**)&h->host_counters, sizeof(DevCounters), hipHostMallocDefault) != hipSuccess) {
    delete h;
    return KGC_E_NOMEM;
  }
  if (hipHostMalloc((void**)&h->host_gstate, sizeof(GroupState), hipHostMallocDefault) != hipSuccess) {
    kgc_destroy(h);
    return KGC_E_NOMEM;
  }
  for (auto& e : h->ev)
    if (hipEventCreate(&e) != hipSuccess) { kgc_destroy(h); return KGC_E_HIP; }
  *out = h;
  return KGC_OK;
}

void kgc_destroy(kgc_handle* h) {
  if (!h) return;
  for (DevBuf* b : {&h->slot_ent, &h->opB, &h->opA, &h->normsB, &h->normsA, &h->counters, &h->params,
                    &h->gstate, &h->unc_a, &h->unc_b, &h->group_of, &h->piv_ent, &h->best, &h->gsize, &h->goff, &h->gfill,
                    &h->cent, &h->rad, &h->bitmap, &h->row_start, &h->row_count, &h->cols, &h->active_rows, &h->cnorm,
                    &h->gram, &h->relu, &h->reln, &h->asg_a, &h->asg_b, &h->limr, &h->top1_buf, &h->top1_state,
                    &h->unit_first, &h->unit_n, &h->cent_u, &h->rad_u, &h->cnorm_u, &h->gram_u, &h->relu_u, &h->pair_list,
                    &h->pair_count, &h->xlist, &h->tile_rows, &h->se_a, &h->se_b, &h->zero_row, &h->cent_a, &h->rad_a, &h->top1_a, &h->top1_b, &h->top1_pick, &h->top_samples, &h->topk_state})
    release(*b);
  if (h->host_gstate) (void)hipHostFree(h->host_gstate);
  if (h->host_counters) (void)hipHostFree(h->host_counters);
  for (auto& e : h->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : h->join_ev)
    if (e) (void)hipEventDestroy(e);
  delete h;
}

const char* kgc_last_error(const kgc_handle* h) { return h ? h->err.c_str() : "null handle"; }

int kgc_join_ab(kgc_handle* hd, const void* A, const void* B, int64_t N, int32_t d, int32_t R, int32_t b_per_relation,
                int32_t p, float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count) {
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  hd->prep.valid = false;            // (this call overwrites what a join over blocks keeps in the handle)
  int rc = check_common(hd, A, N, d, B, R);
  if (rc != KGC_OK) return rc;
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (std::isnan(delta)) return fail(hd, KGC_E_INVALID, "delta is NaN");
  if (cap > 0 && !out_triples) return fail(hd, KGC_E_INVALID, "out_triples is NULL with cap > 0");
  if ((uintptr_t)out_triples % 16) return fail(hd, KGC_E_INVALID, "out_triples must be 16-byte aligned");
  hd->err.clear();
  hd->stats = kgc_stats{};
  hd->stats.triples_total = (uint64_t)N * (uint64_t)N * (uint64_t)R;
  if (N == 0 || R == 0) return KGC_OK;

  hipStream_t st = hd->stream;
  const int dtype = hd->cfg.dtype;
  const size_t esz = dtype == KGC_BF16 ? 2 : 4;
  const bool prune = hd->cfg.prune != KGC_PRUNE_OFF && delta >= 0.f;
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  const int k16 = (d + kNormCols + 15) / 16;
  // the kernels of kgc_join: dense, or (pruned) walking the tile lists
  int tile_id;
  if (prune) tile_id = pruned_l2_tile(N, KS, kDefaultL2Tile);
  else tile_id = KS <= kDirectMaxKS ? kDenseL2Tile : KS <= kDirectHalfMaxKS ? kDirectHalfL2Tile : kDefaultL2Tile;
  const TileCfg tc = kL2Tiles[tile_id];
  // pruned L2 joins on the 128 x 128 head-resident tiles may go tile by tile instead (decided per batch on the device)
  const bool pairs_ok = prune && p == 2 && tile_id == kResidentL2Tile;
  const int BM = (p == 2) ? tc.bm : kL1Tile, BN = (p == 2) ? tc.bn : kL1Tile;
  if ((rc = ensure(hd, hd->counters, sizeof(DevCounters))) || (rc = ensure(hd, hd->params, sizeof(JoinParams))) ||
      (rc = ensure(hd, hd->zero_row, (size_t)d * 4)))
    return rc;
  DevCounters* cnt = (DevCounters*)hd->counters.p;
  JoinParams* prm = (JoinParams*)hd->params.p;
  while (hd->join_ev.size() < 2) {
    hipEvent_t e;
    KGC_HIP(hd, hipEventCreate(&e));
    hd->join_ev.push_back(e);
  }
  KGC_HIP(hd, hipEventRecord(hd->ev[0], st));
  k_fill_u32<<<grid_for(sizeof(DevCounters) / 4, 256), 256, 0, st>>>((uint32_t*)cnt, sizeof(DevCounters) / 4, 0u);
  k_fill_u32<<<grid_for(d, 256), 256, 0, st>>>((uint32_t*)hd->zero_row.p, d, 0u);

  // Row order.  Pruned: the rows of B (of its first relation) are grouped as the entities of kgc_join are, and every
  // relation's A[r] and B[r] are summarised in that order: connectors are maps of one entity set, so rows that are
  // close in B[0] tend to be close in the others; where they are not, the radii grow and less is pruned, never more.
  int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  uint64_t n_groups = 0;
  if (prune) {
    UnitTable unused{};
    if ((rc = group_rows(hd, B, N, d, p, delta, KS, k16, &Nslots, &n_groups, &unused)) != KGC_OK) return rc;
  } else {
    if ((rc = ensure(hd, hd->slot_ent, Nslots * 4))) return rc;
    k_identity_slots<<<grid_for(Nslots, 256), 256, 0, st>>>((int32_t*)hd->slot_ent.p, N, Nslots);
  }
  const int32_t* slot_ent = (const int32_t*)hd->slot_ent.p;
  const int nH = (int)(Nslots / BM), nT = (int)(Nslots / BN);
  const int64_t n_micro = Nslots / kMicro;
  const int words_per_row = (nT + 31) / 32;
  const int64_t tiles_per_rel = (int64_t)nH * nT;
  if (nH > 65535 && p == 1 && !prune) return fail(hd, KGC_E_INVALID, "N too large for one launch grid");
  if (prune && tiles_per_rel > kMaxTileList) return fail(hd, KGC_E_INVALID, "N too large for the pruned tile list");
  const size_t op_bytes = (size_t)KS * Nslots * kSliceK * 2;
  KGC_HIP(hd, hipEventRecord(hd->join_ev[0], st));

  RecheckCtx cx{};
  cx.E = A; cx.Et = B; cx.hstride = (int64_t)N * d; cx.tstride = b_per_relation ? (int64_t)N * d : 0;
  cx.Rv = hd->zero_row.p; cx.rstride = 0;             // the head rows already are connector_1(h, r)
  cx.slot_ent = slot_ent; cx.slot_ent_t = slot_ent; cx.dtype = dtype; cx.d = d; cx.p = p; cx.delta = (double)delta;
  cx.out = out_triples; cx.cap = cap; cx.hit_counter = &cnt->hits; cx.cand_counter = &cnt->candidates; cx.no_self = 0;
  set_alignment(cx);
  const size_t stage_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
  // relation batches: the staged operands, the summaries and the tile lists of a batch must fit the workspace
  const int64_t ws = hd->cfg.workspace_bytes > 0 ? hd->cfg.workspace_bytes : kDefaultWorkspace;
  int64_t RBmax = std::min<int64_t>(R, 65535);
  if (p == 2) RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, ws / (int64_t)(op_bytes * (b_per_relation ? 2 : 1))));
  if (prune) {
    RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, kMaxTileList / tiles_per_rel));
    RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, ws / (int64_t)((size_t)n_micro * d * 4 * 2)));
  }
  if (p == 2 && ((rc = ensure(hd, hd->opA, op_bytes * (size_t)RBmax)) ||
                 (rc = ensure(hd, hd->opB, op_bytes * (size_t)(b_per_relation ? RBmax : 1)))))
    return rc;
  const int64_t nb_sum = b_per_relation ? RBmax : 1;        // tail summaries held at a time
  if (prune && ((rc = ensure(hd, hd->cent, (size_t)nb_sum * n_micro * d * 4)) || (rc = ensure(hd, hd->rad, (size_t)nb_sum * n_micro * 4)) ||
                (rc = ensure(hd, hd->cnorm, (size_t)RBmax * n_micro * 4)) ||
                (rc = ensure(hd, hd->cent_a, (size_t)RBmax * n_micro * d * 4)) || (rc = ensure(hd, hd->rad_a, (size_t)RBmax * n_micro * 4)) ||
                (rc = ensure(hd, hd->bitmap, (size_t)RBmax * nH * words_per_row * 4)) ||
                (rc = ensure(hd, hd->row_start, (size_t)RBmax * nH * 4)) || (rc = ensure(hd, hd->row_count, (size_t)RBmax * nH * 4)) ||
                (rc = ensure(hd, hd->cols, (size_t)RBmax * tiles_per_rel * 4)) ||
                (pairs_ok && (rc = ensure(hd, hd->tile_rows, (size_t)RBmax * tiles_per_rel * 4))) ||
                (rc = ensure(hd, hd->active_rows, (size_t)RBmax * nH * 4))))
    return rc;
  const unsigned row_grid_max = 4096;
  int nbatch = 0;
  for (int64_t r0 = 0; r0 < R; r0 += RBmax, ++nbatch) {
    const int RB = (int)std::min<int64_t>(RBmax, R - r0);
    const uint32_t* active_rows = nullptr;
    const unsigned int* n_active = nullptr;
    if (prune) {
      // summaries of the batch's A[r] (and B[r]) rows in slot order, bound on micro-tile pairs, tile lists
      if (b_per_relation || r0 == 0) {
        if (p == 2)
          k_micro_summary<2><<<dim3((unsigned)n_micro, (unsigned)(b_per_relation ? RB : 1), 1), 64, 0, st>>>(
              B, dtype, d, slot_ent, n_micro, (float*)hd->cent.p, (float*)hd->rad.p, (float*)hd->cnorm.p,
              b_per_relation ? (int)r0 : 0, b_per_relation ? (int64_t)N * d : 0);
        else
          k_micro_summary<1><<<dim3((unsigned)n_micro, (unsigned)(b_per_relation ? RB : 1), 1), 64, 0, st>>>(
              B, dtype, d, slot_ent, n_micro, (float*)hd->cent.p, (float*)hd->rad.p, (float*)hd->cnorm.p,
              b_per_relation ? (int)r0 : 0, b_per_relation ? (int64_t)N * d : 0);
      }
      if (p == 2)
        k_micro_summary<2><<<dim3((unsigned)n_micro, (unsigned)RB, 1), 64, 0, st>>>(
            A, dtype, d, slot_ent, n_micro, (float*)hd->cent_a.p, (float*)hd->rad_a.p, (float*)hd->cnorm.p, (int)r0, (int64_t)N * d);
      else
        k_micro_summary<1><<<dim3((unsigned)n_micro, (unsigned)RB, 1), 64, 0, st>>>(
            A, dtype, d, slot_ent, n_micro, (float*)hd->cent_a.p, (float*)hd->rad_a.p, (float*)hd->cnorm.p, (int)r0, (int64_t)N * d);
      const int64_t bm_words = (int64_t)RB * nH * words_per_row;
      k_fill_u32<<<grid_for(bm_words, 256), 256, 0, st>>>((uint32_t*)hd->bitmap.p, bm_words, 0u);
      TileDistArgs ta{};
      ta.X = hd->cent_a.p; ta.dtypeX = KGC_F32; ta.n_rows = n_micro; ta.Y = hd->cent.p; ta.dtypeY = KGC_F32; ta.n_cols = n_micro;
      ta.shift = nullptr; ta.dtype_shift = KGC_F32; ta.r0 = 0; ta.d = d;
      ta.rad = (const float*)hd->rad.p; ta.rad_rows = (const float*)hd->rad_a.p; ta.x_rel_rows = n_micro;
      ta.y_rel_rows = b_per_relation ? n_micro : 0;
      ta.delta = delta; ta.bitmap = (uint32_t*)hd->bitmap.p; ta.nH = nH; ta.words_per_row = words_per_row;
      ta.micro_per_bm = BM / kMicro; ta.micro_per_bn = BN / kMicro;
      const dim3 g((unsigned)((n_micro + 127) / 128), (unsigned)((n_micro + 127) / 128), (unsigned)RB);
      if (p == 2) k_tile_dist<2, kEpiBound><<<g, 256, 0, st>>>(ta);
      else k_tile_dist<1, kEpiBound><<<g, 256, 0, st>>>(ta);
      k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)&cnt->tile_cursor, 3, 0u);      // cursor and n_active
      k_rows_from_bitmap<<<(unsigned)(((int64_t)RB * nH + 256 * bitmap_rows_per_lane(words_per_row) - 1) / (256 * bitmap_rows_per_lane(words_per_row))), 256, 0, st>>>(
          (const uint32_t*)hd->bitmap.p, words_per_row, (int64_t)RB * nH, (uint32_t*)hd->row_start.p,
          (uint32_t*)hd->row_count.p, (uint32_t*)hd->cols.p, &cnt->tile_cursor, (uint32_t*)hd->active_rows.p, &cnt->n_active,
          pairs_ok ? (uint32_t*)hd->tile_rows.p : nullptr);
      k_batch_tiles<<<1, 64, 0, st>>>(cnt, pairs_ok ? 1 : 0, 0, 0ull, 0ull);
      active_rows = (const uint32_t*)hd->active_rows.p;
      n_active = &cnt->n_active;
    }
    const unsigned row_grid = (unsigned)std::min<int64_t>((int64_t)RB * nH, row_grid_max);
    if (p == 2) {
      const int stage_all = grid_for((int64_t)RB * (Nslots / kStageRows), 1);
      if (b_per_relation)
        k_stage_operands<false><<<stage_all, 256, stage_lds, st>>>(B, nullptr, dtype, d, (int)r0, RB, slot_ent, Nslots, KS,
                                                                 (uint16_t*)hd->opB.p, nullptr, cnt->max_b, nullptr, nullptr, 0,
                                                                 kStageRows, (int64_t)N * d, nullptr, delta);
      else if (r0 == 0)
        k_stage_operands<false><<<grid_for(Nslots / kStageRows, 1), 256, stage_lds, st>>>(
            B, nullptr, dtype, d, 0, 1, slot_ent, Nslots, KS, (uint16_t*)hd->opB.p, nullptr, cnt->max_b, nullptr, nullptr, 0,
            kStageRows, 0, nullptr, delta);
      // head rows: all of them (dense), or those of the head tiles that still have tail tiles (pruned)
      const int stage_a = prune ? (int)std::min<int64_t>((int64_t)RB * nH * (BM / kStageRows), 4096) : stage_all;
      k_stage_operands<true><<<stage_a, 256, stage_lds, st>>>(A, nullptr, dtype, d, (int)r0, RB, slot_ent, Nslots, KS,
                                                             (uint16_t*)hd->opA.p, nullptr, cnt->max_a, active_rows, n_active, nH, BM,
                                                             (int64_t)N * d, nullptr, delta);
      // the maxima only grow from batch to batch: the filter threshold stays on the safe side
      k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, KS * kSliceK);
      JoinStreamArgs sa{};
      sa.A = (const uint16_t*)hd->opA.p; sa.B = (const uint16_t*)hd->opB.p; sa.prm = prm; sa.Nslots = Nslots;
      sa.KS = KS; sa.k16 = k16; sa.nH = nH; sa.nT = nT; sa.r0 = (int)r0; sa.RB = RB; sa.b_per_rel = b_per_relation ? 1 : 0;
      sa.cx = cx;
      void (*kern)(const JoinStreamArgs) = prune ? tc.listed_kernel : tc.stream_kernel;
      if (tile_id == kDenseL2Tile) kern = dense_kernel_for(k16);
      size_t dyn_lds = 0;
      if (tc.head_resident) {
        dyn_lds = ((size_t)KS * BM + (size_t)tc.tail_buffers * BN) * kSliceK * 2;
        if (prune && tc.tail_buffers == 0) {      // the barrier-free form keeps a row's tile list behind the head slices, in segments if need be
          if (dyn_lds + 1024 > kMaxLds) return fail(hd, KGC_E_INVALID, "d too large for the pruned barrier-free tile variant");
          sa.cols_lds = (int)std::min<size_t>((kMaxLds - dyn_lds) / 4, (size_t)nT);
          if (hd->list_seg_cap > 0) sa.cols_lds = std::min(sa.cols_lds, hd->list_seg_cap);
          dyn_lds += (size_t)sa.cols_lds * 4;
        }
        if (prune && tc.tail_buffers > 0) {
          const size_t spare = kMaxLds / tc.blocks_per_cu - (dyn_lds + tc.static_lds);
          sa.cols_lds = (int)std::min<size_t>(spare / 4, (size_t)nT);
          if (sa.cols_lds < nT) sa.cols_lds = 0;
          dyn_lds += (size_t)sa.cols_lds * 4;
        }
        KGC_HIP(hd, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds));
      }
      const bool lists_blocks = tile_id != kDenseL2Tile && tile_id != kDirectL2Tile && tile_id != kDirectHalfL2Tile;
      if (lists_blocks) {
        if ((rc = ensure(hd, hd->xlist, (size_t)hd->xcap * sizeof(ExactEntry)))) return rc;
        sa.xlist = (ExactEntry*)hd->xlist.p; sa.xcount = &cnt->n_exact; sa.xcap = hd->xcap;
      }
      if (prune) {
        sa.row_start = (const uint32_t*)hd->row_start.p; sa.row_count = (const uint32_t*)hd->row_count.p;
        sa.cols = (const uint32_t*)hd->cols.p; sa.active_rows = active_rows; sa.n_active = n_active;
        if (pairs_ok) { sa.tile_rows = (const uint32_t*)hd->tile_rows.p; sa.tile_total = &cnt->tile_cursor; sa.pair_mode = &cnt->pair_mode; }
        hipLaunchKernelGGL(kern, dim3(tile_id == kDirectL2Tile ? (row_grid + 255u) & ~255u : row_grid, 1, 1), dim3(tc.threads), dyn_lds, st, sa);
        if (pairs_ok) {
          const size_t pair_lds = (size_t)2 * KS * 128 * kSliceK * 2;
          KGC_HIP(hd, hipFuncSetAttribute((const void*)k_join_l2_pairs, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pair_lds));
          hipLaunchKernelGGL(k_join_l2_pairs, dim3(hd->pairs_grid), dim3(256), pair_lds, st, sa);      // two resident blocks per compute unit, each walks its tiles
        }
      } else {
        const int64_t tile_bytes = (int64_t)BN * KS * kSliceK * 2;
        const int64_t range_bytes = tc.head_resident ? resident_range_bytes(nT * tile_bytes) : kL2RangeBytes;
        int64_t nsplit = (nT * tile_bytes + range_bytes - 1) / range_bytes;
        nsplit = std::max<int64_t>(nsplit, (4096 + (int64_t)nH * RB - 1) / ((int64_t)nH * RB));
        nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, std::min<int64_t>(nT, 65535)));
        hipLaunchKernelGGL(kern, dim3((unsigned)nH, (unsigned)RB, (unsigned)nsplit), dim3(tc.threads), dyn_lds, st, sa);
      }
      if (lists_blocks) {      // the exact stage of what the launch listed, then an empty list for the next batch
        launch_exact_blocks(st, (const ExactEntry*)hd->xlist.p, &cnt->n_exact, hd->xcap, &cnt->exact_total, &cnt->exact_need, cx);
        k_fill_u32<<<1, 64, 0, st>>>(&cnt->n_exact, 1, 0u);
      }
    } else {
      k_row_l1_max<<<grid_for((int64_t)RB * N * 32, 256), 256, 0, st>>>((const char*)A + (size_t)r0 * N * d * esz, (int64_t)RB * N, d,
                                                                    dtype, cnt->max_a);
      if (b_per_relation || r0 == 0)
        k_row_l1_max<<<grid_for((int64_t)(b_per_relation ? RB : 1) * N * 32, 256), 256, 0, st>>>(
            (const char*)B + (b_per_relation ? (size_t)r0 * N * d * esz : 0), (int64_t)(b_per_relation ? RB : 1) * N, d, dtype,
            cnt->max_b);
      k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, 0);
      JoinL1Args la{};
      la.prm = prm; la.Nslots = Nslots; la.nH = nH; la.nT = nT; la.r0 = (int)r0; la.RB = RB; la.cx = cx;
      if (prune) {
        la.row_start = (const uint32_t*)hd->row_start.p; la.row_count = (const uint32_t*)hd->row_count.p;
        la.cols = (const uint32_t*)hd->cols.p; la.active_rows = active_rows; la.n_active = n_active;
        hipLaunchKernelGGL(k_join_l1, dim3(row_grid, 1, 1), dim3(256), 0, st, la);
      } else {
        hipLaunchKernelGGL(k_join_l1, dim3((unsigned)nT, (unsigned)nH, (unsigned)RB), dim3(256), 0, st, la);
      }
    }
    hd->stats.join_launches++;
  }
  KGC_HIP(hd, hipEventRecord(hd->join_ev[1], st));
  KGC_HIP(hd, hipGetLastError());
  KGC_HIP(hd, hipMemcpyAsync(hd->host_counters, cnt, 48, hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipEventRecord(hd->ev[2], st));
  KGC_HIP(hd, wait_event(hd->ev[2]));

  // A batch that wanted to list more accumulator blocks than the list holds has dropped the rest (and counted
  // them): the list grows to what was asked for and the join runs again from the start.
  if (hd->host_counters->exact_need > hd->xcap) {
    const unsigned long long need = hd->host_counters->exact_need;
    hd->xcap = (unsigned int)std::min<unsigned long long>(need + need / 4 + 1024, 0xffffffffull);
    return kgc_join_ab(hd, A, B, N, d, R, b_per_relation, p, delta, out_triples, cap, count);
  }

  kgc_stats& s = hd->stats;
  s.emitted = hd->host_counters->hits;
  s.candidates = hd->host_counters->candidates;
  s.tiles_total = (uint64_t)tiles_per_rel * (uint64_t)R;
  s.tiles_evaluated = prune ? hd->host_counters->tiles : s.tiles_total;
  s.tiles_pruned = s.tiles_total - s.tiles_evaluated;
  s.pairs_evaluated = prune ? s.tiles_evaluated * (uint64_t)BM * (uint64_t)BN : s.triples_total;
  s.groups = n_groups;
  s.tile_m = BM; s.tile_n = BN;
  s.k_padded = (p == 2) ? k16 * 16 : d;
  s.relation_batches = nbatch;
  s.join_variant = (p == 2) ? tile_id + 1 : 0;
  s.exact_blocks = (int32_t)std::min<unsigned long long>(hd->host_counters->exact_total, 2147483647ull);
  (void)hipEventElapsedTime(&s.ms_total, hd->ev[0], hd->ev[2]);
  (void)hipEventElapsedTime(&s.ms_join, hd->join_ev[0], hd->join_ev[1]);   // staging, summaries and bound of each batch included
  s.ms_precompute = s.ms_total - s.ms_join;
  *count = s.emitted;
  return s.emitted > cap ? KGC_OVERFLOW : KGC_OK;
}


// The structured-embedding instance of the general form (Section 4.3): a = W_lhs[r] h, b = W_rhs[r] t.  The
// connector rows of a relation batch are formed here, in float32 (a tiled float32 product: the chip's float32 vector
// and matrix rates are the same, and the exact stage needs every bit of them), into the handle's own buffers, and the
// batch then runs through kgc_join_ab on those rows; its records get the batch's first relation added.
int kgc_join_se(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* W_lhs, const void* W_rhs, int32_t R,
                int32_t p, float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count) {
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  if (N < 0 || R < 0 || d < 1) return fail(hd, KGC_E_INVALID, "negative size or d < 1");
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (cap > 0 && !out_triples) return fail(hd, KGC_E_INVALID, "out_triples is NULL but cap > 0");
  if (N == 0 || R == 0) { hd->stats = kgc_stats{}; return KGC_OK; }
  if (!E || !W_lhs || !W_rhs) return fail(hd, KGC_E_INVALID, "E, W_lhs or W_rhs is NULL");
  if (hd->static_mode) return fail(hd, KGC_E_INVALID, "kgc_join_se allocates: not available inside kgc_join_static");
  hipStream_t st = hd->stream;
  const int dtype = hd->cfg.dtype;
  // connector rows of as many relations as fit half the workspace (both sides, float32), at most 4 GiB a side
  const int64_t ws = hd->cfg.workspace_bytes > 0 ? hd->cfg.workspace_bytes : kDefaultWorkspace;
  const int64_t per_rel = (int64_t)N * d * 4;
  const int64_t RB_max = std::max<int64_t>(1, std::min<int64_t>({(int64_t)R, (ws / 4) / per_rel, (4ll << 30) / per_rel}));
  int rc;
  if ((rc = ensure(hd, hd->se_a, (size_t)RB_max * per_rel)) || (rc = ensure(hd, hd->se_b, (size_t)RB_max * per_rel))) return rc;
  kgc_stats total{};
  uint64_t found = 0, written = 0;
  const size_t esz = dtype == KGC_BF16 ? 2 : 4;
  int batches = 0;
  for (int64_t r0 = 0; r0 < R; r0 += RB_max, ++batches) {
    const int RB = (int)std::min<int64_t>(RB_max, R - r0);
    for (int side = 0; side < 2; ++side) {
      TileDistArgs td{};
      td.X = E; td.dtypeX = dtype; td.n_rows = N;
      td.Y = (const char*)(side ? W_rhs : W_lhs) + (size_t)r0 * d * d * esz; td.dtypeY = dtype; td.n_cols = d;
      td.y_rel_rows = d; td.shift = nullptr; td.dtype_shift = dtype; td.d = d;
      td.matrix = (float*)(side ? hd->se_b.p : hd->se_a.p); td.matrix_rel_stride = (int64_t)N * d;
      k_tile_dist<0, kEpiMatrix><<<dim3((unsigned)((d + 127) / 128), (unsigned)((N + 127) / 128), (unsigned)RB), 256, 0, st>>>(td);
    }
    KGC_HIP(hd, hipGetLastError());
    // the batch through the general form, on float32 rows whatever the handle's storage type
    const int32_t keep_dtype = hd->cfg.dtype;
    hd->cfg.dtype = KGC_F32;
    uint64_t c = 0;
    rc = kgc_join_ab(hd, hd->se_a.p, hd->se_b.p, N, d, RB, 1, p, delta, out_triples ? out_triples + written : nullptr,
                     cap - written, &c);
    hd->cfg.dtype = keep_dtype;
    if (rc != KGC_OK && rc != KGC_OVERFLOW) return rc;
    const uint64_t kept = std::min<uint64_t>(c, cap - written);
    if (kept > 0 && r0 > 0) k_shift_relation<<<grid_for((int64_t)kept, 256), 256, 0, st>>>(out_triples + written, kept, (int32_t)r0);
    found += c; written += kept;
    const kgc_stats& b = hd->stats;
    total.tiles_total += b.tiles_total; total.tiles_evaluated += b.tiles_evaluated; total.tiles_pruned += b.tiles_pruned;
    total.pairs_evaluated += b.pairs_evaluated; total.candidates += b.candidates; total.join_launches += b.join_launches;
    total.ms_total += b.ms_total; total.ms_precompute += b.ms_precompute; total.ms_prune += b.ms_prune; total.ms_join += b.ms_join;
    total.relation_batches += b.relation_batches; total.exact_blocks += b.exact_blocks;
    total.groups = b.groups; total.tile_m = b.tile_m; total.tile_n = b.tile_n; total.k_padded = b.k_padded; total.join_variant = b.join_variant;
  }
  KGC_HIP(hd, hipStreamSynchronize(st));
  total.triples_total = (uint64_t)N * (uint64_t)N * (uint64_t)R;
  total.emitted = found;
  hd->stats = total;
  *count = found;
  return found > cap ? KGC_OVERFLOW : KGC_OK;
}

}  // extern "C"

namespace {
// Row order for pruning: entities grouped around local pivots (see kgc_prune.h), groups laid out as runs of slots.
// Fills hd->slot_ent, reads back the number of slots, the number of groups and the unit table of the two-level
// bound test.  `rows` is the N x d array that is grouped (the entity array of kgc_join).
int group_rows(kgc_handle* hd, const void* E, int64_t N, int32_t d, int32_t p, float delta, int KS, int k16, int64_t* Nslots_out,
               uint64_t* n_groups_out, UnitTable* ut_out) {
  int rc;
  hipStream_t st = hd->stream;
  const int dtype = hd->cfg.dtype;
  int64_t Nslots = 0;
  uint64_t n_groups = 0;
  UnitTable ut{};
  // worst case: every group of kSmallGroup rows is padded to a micro-tile
  const int64_t max_padded_groups = std::min<int64_t>(kMaxGroups, N / kSmallGroup + 1);
  const int64_t slots_cap = ((N + (kMicro - 1) * max_padded_groups) + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  if ((rc = ensure(hd, hd->slot_ent, slots_cap * 4)) || (rc = ensure(hd, hd->gstate, sizeof(GroupState))) ||
      (rc = ensure(hd, hd->unc_a, N * 4)) || (rc = ensure(hd, hd->unc_b, N * 4)) ||
      (rc = ensure(hd, hd->group_of, N * 4)) || (rc = ensure(hd, hd->piv_ent, kPivotsPerRound * 4)) ||
      (rc = ensure(hd, hd->best, N * 8)) || (rc = ensure(hd, hd->gsize, kMaxGroups * 4)) ||
      (rc = ensure(hd, hd->goff, kMaxGroups * 4)) || (rc = ensure(hd, hd->gfill, kMaxGroups * 4)) ||
      (rc = ensure(hd, hd->unit_first, kMaxGroups * 4)) || (rc = ensure(hd, hd->unit_n, kMaxGroups * 4)))
    return rc;
  GroupState* gs = (GroupState*)hd->gstate.p;
  int32_t* unc = (int32_t*)hd->unc_a.p;
  int32_t* unc_next = (int32_t*)hd->unc_b.p;
  const float radius_mult = hd->cfg.group_radius > 0.f ? hd->cfg.group_radius : 2.0f;
  float tau = delta > 0.f ? radius_mult * delta : 0.f;
  const int gN = grid_for(std::max<int64_t>(N, kPivotsPerRound), 256);
  // With a head tile that fits in LDS (d <= 602) the rows-against-pivots distances of every round run on the
  // matrix pipes, as a join of all entities (heads, staged once in identity order) with the round's pivots
  // (tails) whose epilogue keeps, per entity, the lowest pivot position within tau.  Otherwise (large d)
  // the float32 vector kernel does it.  Which member of a cluster ends up with which pivot does not touch
  // the result: centres and radii are taken from the rows after the layout.
  // An L1 join is grouped in L2 as well: for differences with independent, similarly sized components
  // ||x||_1 is about sqrt(2 / pi) sqrt(d) ||x||_2, so the L1 radius tau corresponds to that L2 radius; a
  // different ratio only makes the groups a little larger or smaller.
  const bool mfma_assign = KS <= kDirectHalfMaxKS && delta > 0.f;
  const int abm = KS <= kDirectMaxKS ? 256 : 128;           // head tile height of the assignment kernel
  void (*assign_kernel)(const JoinStreamArgs) =
      abm == 256 ? k_join_l2_direct<256, 2, 4, kEpiAssignMin> : k_join_l2_direct<128, 1, 8, kEpiAssignMin>;
  const int64_t Npad = (N + 255) / 256 * 256;
  const size_t asg_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
  if (mfma_assign) {
    if ((rc = ensure(hd, hd->asg_a, (size_t)KS * Npad * kSliceK * 2)) ||
        (rc = ensure(hd, hd->asg_b, (size_t)KS * kPivotsPerRound * kSliceK * 2)))
      return rc;
    // the heads in identity order
    k_stage_operands<true><<<grid_for(Npad / kStageRows, 1), 256, asg_lds, st>>>(
        E, nullptr, dtype, d, 0, 1, nullptr, Npad, KS, (uint16_t*)hd->asg_a.p, nullptr, nullptr,
        nullptr, nullptr, 0, kStageRows, 0, nullptr, -1.f, N);
    KGC_HIP(hd, hipFuncSetAttribute((const void*)assign_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)((size_t)KS * abm * kSliceK * 2)));
  }
  // A radius far below the spacing of the rows groups nothing: every row then lands in the packed tail region in
  // arbitrary order, micro-tiles mix rows from everywhere and no tile can be pruned.  When more than half of the
  // rows end up there, the grouping is repeated with four times the radius (at most three times): groups of the
  // size of the natural clusters prune well even when delta is much smaller than a cluster.
  for (int attempt = 0;; ++attempt) {
  const float tau_l2 = (p == 2) ? tau : tau / (0.79788456f * std::sqrt((float)d));
  unc = (int32_t*)hd->unc_a.p;
  unc_next = (int32_t*)hd->unc_b.p;
  // Sampling density of the pivots among the still uncovered entities, round by round: 1/16, 1/16, 1/8, 1/8, 1/4,
  // 1/2.  With few entities three rounds at 1/4, 1/2 and 1 reach the same cover (their up to 3 x 4,096 pivots are
  // more than a third of the entities; several pivots in one natural cluster do not split it, the lowest one within
  // reach wins), and each round is five launches that a small join feels.
  const bool few = N <= kFewEntities;
  const int n_rounds = few ? 3 : kGroupRounds;
  for (int round = 0; round < n_rounds; ++round) {
    static const int kShift[kGroupRounds] = {4, 4, 3, 3, 2, 1};
    static const int kShiftFew[3] = {2, 1, 0};
    k_round_begin<<<gN, 256, 0, st>>>(gs, unc, (int32_t*)hd->piv_ent.p, (unsigned long long*)hd->best.p,
                                     few ? kShiftFew[round] : kShift[round], mfma_assign ? 1 : 0, round == 0 ? N : 0,
                                     (int32_t*)hd->group_of.p, round);
    if (mfma_assign) {
      k_stage_operands<false><<<kPivotsPerRound / kStageRows, 256, asg_lds, st>>>(
          E, nullptr, dtype, d, 0, 1, (const int32_t*)hd->piv_ent.p, kPivotsPerRound, KS, (uint16_t*)hd->asg_b.p, nullptr,
          nullptr, nullptr, nullptr, 0, kStageRows, 0, &gs->n_piv);
      JoinStreamArgs sa{};
      sa.A = (const uint16_t*)hd->asg_a.p; sa.B = (const uint16_t*)hd->asg_b.p; sa.prm = nullptr; sa.Nslots = Npad;
      sa.KS = KS; sa.k16 = k16; sa.nH = (int)(Npad / abm); sa.nT = kPivotsPerRound / 256; sa.r0 = 0; sa.RB = 1;
      sa.tail_slots = kPivotsPerRound; sa.tail_rows_dev = &gs->n_piv;
      // bf16 rows move a distance by at most 2^-8 (||e|| + ||pivot||); that much either way is of no concern here
      sa.thr_value = tau_l2 * tau_l2;
      sa.best = (unsigned long long*)hd->best.p; sa.group_of = (const int32_t*)hd->group_of.p; sa.n_heads = N;
      // the pivot tiles are dealt to 1, 2 or 4 blocks per head tile, enough to fill the chip
      const int64_t nHa = Npad / abm;
      const unsigned zsplit = nHa >= 1024 ? 1u : nHa >= 512 ? 2u : 4u;
      hipLaunchKernelGGL(assign_kernel, dim3((unsigned)nHa, 1, zsplit), dim3(512), (size_t)KS * abm * kSliceK * 2, st, sa);
    } else {
      TileDistArgs ta{};
      ta.X = E; ta.dtypeX = dtype; ta.row_ids = unc; ta.n_rows_dev = &gs->n_unc; ta.n_rows = N;
      ta.Y = E; ta.dtypeY = dtype; ta.col_ids = (const int32_t*)hd->piv_ent.p; ta.n_cols_dev = &gs->n_piv;
      ta.n_cols = kPivotsPerRound;
      ta.shift = nullptr; ta.dtype_shift = dtype; ta.r0 = 0; ta.d = d; ta.best = (unsigned long long*)hd->best.p;
      ta.delta = tau;
      const dim3 g((unsigned)((std::min<int64_t>(kPivotsPerRound, N) + 127) / 128), (unsigned)((N + 127) / 128), 1);
      if (p == 2) k_tile_dist<2, kEpiAssign><<<g, 256, 0, st>>>(ta);
      else k_tile_dist<1, kEpiAssign><<<g, 256, 0, st>>>(ta);
    }
    k_round_commit<<<gN, 256, 0, st>>>(gs, unc, (const unsigned long long*)hd->best.p, (int32_t*)hd->group_of.p,
                                      unc_next, mfma_assign ? 1 : 0, round);
    std::swap(unc, unc_next);      // (the next round's start, or k_group_clear after the last, closes this round)
  }
  k_group_clear<<<grid_for(std::max<int64_t>(kMaxGroups, slots_cap), 256), 256, 0, st>>>(
      (int32_t*)hd->gsize.p, (int32_t*)hd->gfill.p, kMaxGroups, (int32_t*)hd->slot_ent.p, slots_cap, gs, n_rounds - 1);
  k_group_hist<<<gN, 256, 0, st>>>((const int32_t*)hd->group_of.p, N, (int32_t*)hd->gsize.p);
  k_group_layout<<<1, 1024, 0, st>>>(gs, (const int32_t*)hd->gsize.p, (int32_t*)hd->goff.p, N, (int)kSlotAlign,
                                     (int32_t*)hd->unit_first.p, (int32_t*)hd->unit_n.p);
  k_scatter_slots<<<gN, 256, 0, st>>>(gs, (const int32_t*)hd->group_of.p, (const int32_t*)hd->goff.p,
                                     (int32_t*)hd->gfill.p, N, (int32_t*)hd->slot_ent.p);
  KGC_HIP(hd, hipGetLastError());
  // the layout decides the number of rows, which sizes every later launch: one small read-back
  KGC_HIP(hd, hipMemcpyAsync(hd->host_gstate, gs, sizeof(GroupState), hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipEventRecord(hd->ev[3], st));
  KGC_HIP(hd, wait_event(hd->ev[3]));
  if (attempt >= 3 || !(tau > 0.f) || (int64_t)hd->host_gstate->tail_fill * 2 <= N) break;
  tau *= 4.f;
  }   // attempts
  Nslots = hd->host_gstate->n_slots;
  n_groups = (uint64_t)hd->host_gstate->n_groups;
  if (Nslots < N || Nslots > slots_cap || Nslots % kSlotAlign) return fail(hd, KGC_E_HIP, "group layout out of range");
  ut.first = (const int32_t*)hd->unit_first.p; ut.n = (const int32_t*)hd->unit_n.p;
  ut.n_big = hd->host_gstate->n_big;
  ut.tail_first = hd->host_gstate->tail_base / kMicro;
  ut.n_units = ut.n_big + (int)(Nslots / kMicro) - ut.tail_first;
  if (ut.n_big < 0 || ut.n_big > kMaxGroups || ut.tail_first < 0 || ut.tail_first > Nslots / kMicro)
    return fail(hd, KGC_E_HIP, "unit table out of range");
  *Nslots_out = Nslots;
  *n_groups_out = n_groups;
  *ut_out = ut;
  return KGC_OK;
}

// kgc_top1 / kgc_topk switch the handle to "no self pairs" around their inner joins; this puts it back on every way out
struct NoSelfScope {
  kgc_handle* h;
  NoSelfScope(kgc_handle* hd, bool on) : h(hd) { h->no_self = on ? 1 : 0; }
  ~NoSelfScope() { h->no_self = 0; }
};
constexpr uint64_t kTopCap = 1u << 20;       // records the inner joins of the top-1 / top-k searches may return
constexpr int kTopSamples = 1 << 16;

// Upper bounds of the smallest eligible distance for kgc_top1 / kgc_topk.  *sample_bound: the smallest of
// kTopSamples sampled triples, scored exactly (its triple is known to qualify); *bound: that, or the tighter bound
// of the sub-sampled dense pass when it applies.  samples (optional, host, kTopSamples doubles) receives every
// sampled distance.
int top_bounds(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t r_begin, int32_t R, int32_t p,
               int32_t exclude_self, const RecheckCtx& cx, double* sample_bound_out, double* bound_out, double* samples) {
  // R counts the relations of the search, r_begin .. r_begin + R - 1
  int rc;
  hipStream_t st = hd->stream;
  hd->prep.valid = false;            // (the search overwrites what a join over blocks keeps in the handle)
  Top1State* ts = (Top1State*)hd->top1_state.p;
  Top1State host{};
  double* dev_samples = nullptr;
  if (samples) {
    if ((rc = ensure(hd, hd->top_samples, (size_t)kTopSamples * 8))) return rc;
    dev_samples = (double*)hd->top_samples.p;
  }
  // 1. an upper bound of the answer: the smallest of 65,536 sampled eligible triples
  const int n_sample = kTopSamples;
  k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)ts, sizeof(Top1State) / 4, 0xffffffffu);
  k_top1_sample<<<grid_for((int64_t)n_sample * 16, 256), 256, 0, st>>>(cx, N, r_begin, R, n_sample, exclude_self ? 1 : 0, ts, dev_samples);
  if (samples) KGC_HIP(hd, hipMemcpyAsync(samples, dev_samples, (size_t)kTopSamples * 8, hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipMemcpyAsync(&host, ts, sizeof(Top1State), hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipStreamSynchronize(st));
  double bound;
  std::memcpy(&bound, &host.sample_min, sizeof(double));
  if (!(bound >= 0.0) || std::isinf(bound)) return fail(hd, KGC_E_INVALID, "non-finite distances: E or Rvecs hold non-finite values");
  const double sample_bound = bound;

  // 1b. (L2, head tile fits in LDS, enough entities)  A random triple is almost never a close one, so the
  //     sampled bound is usually far above the answer, where a join prunes nothing.  A dense pass over a
  //     sub-sample -- up to 8,192 heads x 8,192 other tails x the first 32 relations, the barrier-free kernel
  //     with an epilogue that keeps only the smallest squared distance -- costs about a millisecond and
  //     usually lands within a few tens of percent of the answer.
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  if (KS <= kDirectMaxKS && N >= 1024) {     // (the pass measures in L2; for an L1 search its bound is scaled below)
    const int m = (int)std::min<int64_t>(8192, (N / 2) / 256 * 256);
    const int Rs = (int)std::min<int32_t>(R, 32);
    const int k16 = (d + kNormCols + 15) / 16;
    const size_t op_rows = (size_t)KS * m * kSliceK * 2;
    if ((rc = ensure(hd, hd->top1_pick, (size_t)2 * m * 4)) || (rc = ensure(hd, hd->top1_b, op_rows)) ||
        (rc = ensure(hd, hd->top1_a, op_rows * Rs)))
      return rc;
    DevCounters* cnt = (DevCounters*)hd->counters.p;
    int32_t* heads = (int32_t*)hd->top1_pick.p;
    int32_t* tails = heads + m;
    const size_t stage_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
    k_fill_u32<<<grid_for(sizeof(DevCounters) / 4, 256), 256, 0, st>>>((uint32_t*)cnt, sizeof(DevCounters) / 4, 0u);
    k_top1_pick<<<grid_for(m, 256), 256, 0, st>>>(N, m, heads, tails);
    k_stage_operands<false><<<m / kStageRows, 256, stage_lds, st>>>(E, Rvecs, hd->cfg.dtype, d, 0, 1, tails, m, KS,
                                                               (uint16_t*)hd->top1_b.p, nullptr, cnt->max_b, nullptr, nullptr, 0,
                                                               kStageRows);
    k_stage_operands<true><<<grid_for((int64_t)Rs * (m / kStageRows), 1), 256, stage_lds, st>>>(
        E, Rvecs, hd->cfg.dtype, d, r_begin, Rs, heads, m, KS, (uint16_t*)hd->top1_a.p, nullptr, cnt->max_a, nullptr, nullptr, 0,
        kStageRows);
    JoinStreamArgs sa{};
    sa.A = (const uint16_t*)hd->top1_a.p; sa.B = (const uint16_t*)hd->top1_b.p; sa.prm = nullptr; sa.Nslots = m;
    sa.KS = KS; sa.k16 = k16; sa.nH = m / 256; sa.nT = m / 256; sa.r0 = 0; sa.RB = Rs; sa.thr_value = 0.f;
    sa.best = &ts->sub_min;
    const size_t dyn_lds = (size_t)KS * 256 * kSliceK * 2;
    KGC_HIP(hd, hipFuncSetAttribute((const void*)k_join_l2_direct<256, 2, 4, kEpiMinDist>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds));
    hipLaunchKernelGGL((k_join_l2_direct<256, 2, 4, kEpiMinDist>), dim3((unsigned)(m / 256), (unsigned)Rs, 1), dim3(512), dyn_lds,
                       st, sa);
    k_top1_bound<<<1, 64, 0, st>>>(cnt, hd->cfg.dtype, KS * kSliceK, ts);
    KGC_HIP(hd, hipMemcpyAsync(&host, ts, sizeof(Top1State), hipMemcpyDeviceToHost, st));
    KGC_HIP(hd, hipStreamSynchronize(st));
    // ||x||_1 <= sqrt(d) ||x||_2: the pair that attains the L2 bound is at most that far apart in L1
    const double sub = p == 2 ? host.sub_bound : host.sub_bound * std::sqrt((double)d) * (1.0 + 1e-6);
    if (host.sub_bound >= 0.0 && sub < bound) bound = sub;
  }
  *sample_bound_out = sample_bound;
  *bound_out = bound;
  return KGC_OK;
}
}  // namespace

extern "C" {

int kgc_top1(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
             int32_t exclude_self, kgc_triple* out) {
  if (!hd) return KGC_E_INVALID;
  if (!out) return fail(hd, KGC_E_INVALID, "out is NULL");
  out->h = out->r = out->t = -1;
  out->dist = INFINITY;
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (N == 0 || R == 0 || (exclude_self && N < 2)) return KGC_OK;          // no eligible triple
  hipStream_t st = hd->stream;
  constexpr uint64_t kCap = kTopCap;
  if ((rc = ensure(hd, hd->top1_buf, kCap * sizeof(kgc_triple))) || (rc = ensure(hd, hd->top1_state, sizeof(Top1State))) ||
      (rc = ensure(hd, hd->counters, sizeof(DevCounters))))
    return rc;
  Top1State* ts = (Top1State*)hd->top1_state.p;
  Top1State host{};
  RecheckCtx cx{};
  cx.E = E; cx.Et = E; cx.Rv = Rvecs; cx.rstride = d; cx.hstride = 0; cx.tstride = 0; cx.slot_ent = nullptr; cx.slot_ent_t = nullptr; cx.dtype = hd->cfg.dtype; cx.d = d; cx.p = p;
  set_alignment(cx);

  double sample_bound = 0.0, bound = 0.0;
  if ((rc = top_bounds(hd, E, N, d, Rvecs, 0, R, p, exclude_self, cx, &sample_bound, &bound, nullptr)) != KGC_OK) return rc;

  // 2. Joins with a shrinking threshold: every triple at or below the bound comes back; if there are more
  //    than the buffer holds, the smallest distance among those that did come back is the next bound.  The
  //    bound of step 1b rests on an error analysis instead of an exact distance; should a join at it come
  //    back empty, the search falls back to the sampled bound, whose triple is known to qualify.
  NoSelfScope no_self_scope(hd, exclude_self != 0);
  int rounds = 0;
  for (;; ++rounds) {
    float delta = (float)bound;
    if ((double)delta < bound) delta = std::nextafterf(delta, INFINITY);    // the bounding triple must qualify
    uint64_t count = 0;
    rc = kgc_join(hd, E, N, d, Rvecs, R, p, delta, (kgc_triple*)hd->top1_buf.p, kCap, &count);
    if (rc < 0) return rc;
    if (count == 0) {
      if (bound < sample_bound) { bound = sample_bound; continue; }
      return fail(hd, KGC_E_HIP, "top-1 search lost its bounding triple");
    }
    DevCounters* cnt = (DevCounters*)hd->counters.p;
    k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)ts, sizeof(Top1State) / 4, 0xffffffffu);
    k_top1_min<<<256, 256, 0, st>>>((const kgc_triple*)hd->top1_buf.p, &cnt->hits, kCap, 0, ts);
    k_top1_min<<<256, 256, 0, st>>>((const kgc_triple*)hd->top1_buf.p, &cnt->hits, kCap, 1, ts);
    k_top1_exact<<<1, 64, 0, st>>>(cx, ts);
    KGC_HIP(hd, hipMemcpyAsync(&host, ts, sizeof(Top1State), hipMemcpyDeviceToHost, st));
    KGC_HIP(hd, hipStreamSynchronize(st));
    if (rc == KGC_OK) break;                                // everything at or below the bound was seen
    // overflow: the buffer holds a subset; its minimum bounds the answer from above.  When that does not
    // lower the bound any more (a mass of equal distances), any of them is a smallest distance.
    if (!(host.dist < bound) || rounds >= 40) break;
    bound = host.dist;
  }
  hd->no_self = 0;
  out->r = (int32_t)(uint32_t)(host.key_dr & 0xffffffffull);
  out->h = (int32_t)(uint32_t)(host.key_ht >> 32);
  out->t = (int32_t)(uint32_t)(host.key_ht & 0xffffffffull);
  out->dist = (float)host.dist;
  return KGC_OK;
}

int kgc_topk(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
             int32_t exclude_self, uint64_t k, kgc_triple* out_triples, uint64_t* found) {
  return kgc_topk_range(hd, E, N, d, Rvecs, R, p, exclude_self, 0, R, k, out_triples, found);
}

int kgc_topk_range(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                   int32_t exclude_self, int32_t r_begin, int32_t r_end, uint64_t k, kgc_triple* out_triples, uint64_t* found) {
  if (!hd) return KGC_E_INVALID;
  if (!found) return fail(hd, KGC_E_INVALID, "found is NULL");
  *found = 0;
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
  if (r_begin < 0 || r_end < r_begin || r_end > R) return fail(hd, KGC_E_INVALID, "relation range outside [0, R]");
  const int32_t Rn = r_end - r_begin;
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (k > (uint64_t)kTopSamples) return fail(hd, KGC_E_INVALID, "k is limited to 65536");
  if (k > 0 && !out_triples) return fail(hd, KGC_E_INVALID, "out_triples is NULL with k > 0");
  if ((uintptr_t)out_triples % 16) return fail(hd, KGC_E_INVALID, "out_triples must be 16-byte aligned");
  if (k == 0 || N == 0 || Rn == 0 || (exclude_self && N < 2)) return KGC_OK;
  hipStream_t st = hd->stream;
  if ((rc = ensure(hd, hd->top1_buf, kTopCap * sizeof(kgc_triple))) || (rc = ensure(hd, hd->top1_state, sizeof(Top1State))) ||
      (rc = ensure(hd, hd->topk_state, sizeof(TopkState))) || (rc = ensure(hd, hd->counters, sizeof(DevCounters))))
    return rc;
  RecheckCtx cx{};
  cx.E = E; cx.Et = E; cx.Rv = Rvecs; cx.rstride = d; cx.hstride = 0; cx.tstride = 0; cx.slot_ent = nullptr; cx.slot_ent_t = nullptr;
  cx.dtype = hd->cfg.dtype; cx.d = d; cx.p = p;
  set_alignment(cx);
  const double eligible = (double)N * (double)N * (double)Rn - (exclude_self ? (double)N * (double)Rn : 0.0);

  // thresholds to try: from just above the smallest distance upwards.  The k-th smallest of the sampled
  // distances bounds the k-th smallest of all from above (the sample is drawn with replacement, so on small
  // problems it can hold a triple twice: the loop below then simply goes on growing the threshold).
  std::vector<double> samples(kTopSamples);
  double sample_bound = 0.0, thr = 0.0;
  if ((rc = top_bounds(hd, E, N, d, Rvecs, r_begin, Rn, p, exclude_self, cx, &sample_bound, &thr, samples.data())) != KGC_OK) return rc;
  std::nth_element(samples.begin(), samples.begin() + (size_t)(k - 1), samples.end());
  const double kth_sample = samples[(size_t)(k - 1)];
  const bool take_all = eligible <= (double)kTopCap / 4;       // a small problem: every triple fits the buffer
  double lo = 0.0;                                             // a threshold known to return fewer than k
  bool have_lo = false;
  uint64_t count = 0;
  NoSelfScope no_self_scope(hd, exclude_self != 0);
  for (int rounds = 0;; ++rounds) {
    float delta = take_all ? INFINITY : (float)thr;
    if (!take_all && (double)delta < thr) delta = std::nextafterf(delta, INFINITY);
    rc = kgc_join_range(hd, E, N, d, Rvecs, R, p, delta, r_begin, r_end, (kgc_triple*)hd->top1_buf.p, kTopCap, &count);
    if (rc < 0) return rc;
    if (rounds >= 200) return fail(hd, KGC_E_HIP, "top-k search did not settle");
    const uint64_t want = (double)k < eligible ? k : (uint64_t)eligible;
    if (count < want) {                                        // too few: grow (towards the sampled bound first)
      lo = thr; have_lo = true;
      // 8 % steps near the smallest distance (the counts rise steeply there), larger ones if that drags on
      const double grown = thr > 0.0 ? thr * (rounds < 24 ? 1.08 : 1.5) : (kth_sample > 0.0 ? kth_sample * 0x1p-20 : 1e-30);
      thr = (thr < kth_sample && grown > kth_sample) ? kth_sample : grown;
      continue;
    }
    if (rc == KGC_OVERFLOW) {                                  // at least k, but more than the buffer holds: shrink
      thr = have_lo ? 0.5 * (lo + thr) : 0.5 * thr;
      continue;
    }
    break;
  }
  hd->no_self = 0;

  // the k smallest of the `count` records, by radix select on the distance bits
  DevCounters* cnt = (DevCounters*)hd->counters.p;
  TopkState* tk = (TopkState*)hd->topk_state.p;
  k_topk_init<<<1, 256, 0, st>>>(tk, k);
  for (int shift = 24; shift >= 0; shift -= 8) {
    k_topk_hist<<<256, 256, 0, st>>>((const kgc_triple*)hd->top1_buf.p, &cnt->hits, kTopCap, shift, tk);
    k_topk_digit<<<1, 64, 0, st>>>(shift, tk);
  }
  k_topk_emit<<<256, 256, 0, st>>>((const kgc_triple*)hd->top1_buf.p, &cnt->hits, kTopCap, k, tk, out_triples);
  KGC_HIP(hd, hipGetLastError());
  KGC_HIP(hd, hipStreamSynchronize(st));
  *found = count < k ? count : k;
  return KGC_OK;
}

int kgc_calibrate_mfma(int32_t wave_tile, int32_t feed, int32_t ms_target, void* stream, double* tflops, float* ms) {
  if (wave_tile < 0 || wave_tile > 1 || feed < 0 || feed > 2 || ms_target < 1 || ms_target > 5000 || !tflops || !ms)
    return KGC_E_INVALID;
  hipStream_t st = (hipStream_t)stream;
  // tail rows: seven 32-wide slices (d = 200) of a range of about 3 MiB, as one block of the dense join walks
  CalibArgs ca{};
  ca.slices = 7;
  ca.rows = 27 * 256;
  uint16_t* G = nullptr;
  float* sink = nullptr;
  const int64_t n = (int64_t)ca.slices * ca.rows * 32;
  if (hipMalloc((void**)&G, n * 2) != hipSuccess) return KGC_E_NOMEM;
  if (hipMalloc((void**)&sink, 4096 * 512 * 4) != hipSuccess) { (void)hipFree(G); return KGC_E_NOMEM; }
  ca.G = G;
  ca.sink = sink;
  k_calib_fill<<<1024, 256, 0, st>>>(G, n);
  void (*kern)(const CalibArgs) = nullptr;
  int waves = 8, blocks_of = 8;
  if (wave_tile == 0) kern = feed == 0 ? k_calib_mfma<4, 2, 2, 4, 0> : feed == 1 ? k_calib_mfma<4, 2, 2, 4, 1> : k_calib_mfma<4, 2, 2, 4, 2>;
  else { kern = feed == 0 ? k_calib_mfma<4, 4, 2, 2, 0> : feed == 1 ? k_calib_mfma<4, 4, 2, 2, 1> : k_calib_mfma<4, 4, 2, 2, 2>; waves = 4; blocks_of = 16; }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = KGC_OK;
  float t = 0.f;
  const unsigned grid = 256 * 8;                           // eight blocks per CU, one after the other
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = KGC_E_HIP;
  // a short launch gives the rate, the timed launch is then sized for ms_target
  int iters = 6 * 200;
  for (int pass = 0; pass < 2 && rc == KGC_OK; ++pass) {
    ca.iters = iters;
    if (hipEventRecord(e0, st) != hipSuccess) { rc = KGC_E_HIP; break; }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(waves * 64), 0, st, ca);
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&t, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = KGC_E_HIP; break; }
    if (pass == 0) {
      const double per_iter = (double)t / iters;
      int64_t want = (int64_t)((double)ms_target / (per_iter > 1e-9 ? per_iter : 1e-9));
      want = want / 6 * 6;
      iters = (int)(want < 6 ? 6 : want > (1 << 28) ? (1 << 28) : want);
    }
  }
  if (rc == KGC_OK) {
    const double flop = (double)grid * waves * (double)iters * blocks_of * 32768.0;
    *tflops = flop / ((double)t * 1e-3) / 1e12;
    *ms = t;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(G);
  (void)hipFree(sink);
  return rc;
}

int kgc_get_stats(const kgc_handle* h, kgc_stats* out) {
  if (!h || !out) return KGC_E_INVALID;
  *out = h->stats;
  return KGC_OK;
}

int kgc_norms(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, float* nB,
              float* nA) {
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
  hd->prep.valid = false;
  hd->err.clear();
  if (N == 0) return KGC_OK;
  hipStream_t st = hd->stream;
  const int dtype = hd->cfg.dtype;
  const int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  const size_t op_bytes = (size_t)KS * Nslots * kSliceK * 2;
  if ((rc = ensure(hd, hd->slot_ent, Nslots * 4)) || (rc = ensure(hd, hd->opB, op_bytes)) ||
      (rc = ensure(hd, hd->opA, op_bytes)) || (rc = ensure(hd, hd->normsB, Nslots * 4)))
    return rc;
  k_identity_slots<<<grid_for(Nslots, 256), 256, 0, st>>>((int32_t*)hd->slot_ent.p, N, Nslots);
  const int g = grid_for(Nslots / kStageRows, 1);
  const size_t stage_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
  if (nB) {
    k_stage_operands<false><<<g, 256, stage_lds, st>>>(E, Rvecs, dtype, d, 0, 1, (const int32_t*)hd->slot_ent.p, Nslots, KS,
                                               (uint16_t*)hd->opB.p, (float*)hd->normsB.p, nullptr, nullptr, nullptr, 0, kStageRows);
    k_scatter_norms<<<grid_for(Nslots, 256), 256, 0, st>>>((const float*)hd->normsB.p, (const int32_t*)hd->slot_ent.p,
                                                           Nslots, N, 1, nB);
  }
  if (nA) {
    for (int r = 0; r < R; ++r) {
      k_stage_operands<true><<<g, 256, stage_lds, st>>>(E, Rvecs, dtype, d, r, 1, (const int32_t*)hd->slot_ent.p, Nslots, KS,
                                                (uint16_t*)hd->opA.p, (float*)hd->normsB.p, nullptr, nullptr, nullptr, 0, kStageRows);
      k_scatter_norms<<<grid_for(Nslots, 256), 256, 0, st>>>((const float*)hd->normsB.p,
                                                             (const int32_t*)hd->slot_ent.p, Nslots, N, 1,
                                                             nA + (int64_t)r * N);
    }
  }
  KGC_HIP(hd, hipGetLastError());
  KGC_HIP(hd, hipStreamSynchronize(st));
  return KGC_OK;
}

int kgc_join(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
             float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count) {
  return kgc_join_range(hd, E, N, d, Rvecs, R, p, delta, 0, R, out_triples, cap, count);
}

int kgc_join_static(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                    float delta, kgc_triple* out_triples, uint64_t cap, uint64_t* count) {
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (hd->cfg.factorised) return fail(hd, KGC_E_INVALID, "kgc_join_static: not with the factorised kernel");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != hd->device)
    return fail(hd, KGC_E_INVALID, "kgc_join_static: the handle's device is not the current device");
  void* base = nullptr;
  if ((rc = static_scratch_ptr(dev, &base)) != KGC_OK) return fail(hd, rc, "kgc_join_static: no static scratch on this device");

  // Layout of the dense join's scratch inside the static array (the sizes kgc_join_range asks for with pruning off):
  // counters, threshold, slot order, tail operands and norms, then as many relations' head operands as fit.
  const int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  const size_t op_rel = (p == 2) ? (size_t)KS * Nslots * kSliceK * 2 : 0;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off = 0;
  auto carve = [&](size_t bytes) { const size_t o = off; off += up(bytes ? bytes : 256); return o; };
  const size_t o_cnt = carve(sizeof(DevCounters)), o_prm = carve(sizeof(JoinParams)), o_slot = carve((size_t)Nslots * 4);
  const size_t o_opB = carve(op_rel), o_nB = carve(p == 2 ? (size_t)Nslots * 4 : 0);
  const size_t per_rel = up(op_rel) + up((size_t)Nslots * 4);           // staged head operands and their norms
  int64_t RB = 0;
  if (off < kStaticScratchBytes) RB = (int64_t)((kStaticScratchBytes - off) / (p == 2 ? per_rel : 1));
  if (p == 2 && RB > R) RB = R;
  if (off >= kStaticScratchBytes || (p == 2 && R > 0 && RB < 1)) {
    char msg[200];
    std::snprintf(msg, sizeof msg, "kgc_join_static: N = %lld, d = %d need more than the %zu MiB of static scratch",
                  (long long)N, (int)d, kStaticScratchBytes >> 20);
    return fail(hd, KGC_E_INVALID, msg);
  }
  const size_t o_opA = carve(p == 2 ? op_rel * (size_t)RB : 0), o_nA = carve(p == 2 ? (size_t)RB * Nslots * 4 : 0);
  if (off > kStaticScratchBytes) return fail(hd, KGC_E_INVALID, "kgc_join_static: layout exceeds the static scratch");

  // the handle's buffers point into the array for the duration of the call; nothing on this path may allocate
  struct Swap {
    kgc_handle* h;
    DevBuf counters, params, slot_ent, opB, normsB, opA, normsA;
    kgc_config cfg;
    explicit Swap(kgc_handle* hd)
        : h(hd), counters(hd->counters), params(hd->params), slot_ent(hd->slot_ent), opB(hd->opB), normsB(hd->normsB),
          opA(hd->opA), normsA(hd->normsA), cfg(hd->cfg) {}
    ~Swap() {
      h->counters = counters; h->params = params; h->slot_ent = slot_ent; h->opB = opB; h->normsB = normsB;
      h->opA = opA; h->normsA = normsA; h->cfg = cfg; h->static_mode = false; h->ws_override = 0;
    }
  } swap(hd);
  char* b = (char*)base;
  auto at = [&](size_t o, size_t bytes) { DevBuf v; v.p = b + o; v.bytes = up(bytes ? bytes : 256); return v; };
  hd->counters = at(o_cnt, sizeof(DevCounters)); hd->params = at(o_prm, sizeof(JoinParams));
  hd->slot_ent = at(o_slot, (size_t)Nslots * 4);
  hd->opB = at(o_opB, op_rel); hd->normsB = at(o_nB, (size_t)Nslots * 4);
  hd->opA = at(o_opA, op_rel * (size_t)RB); hd->normsA = at(o_nA, (size_t)RB * Nslots * 4);
  hd->cfg.prune = KGC_PRUNE_OFF;
  hd->static_mode = true;
  hd->ws_override = p == 2 ? (int64_t)RB * (int64_t)(op_rel + (size_t)Nslots * 4) : 0;
  return kgc_join_range(hd, E, N, d, Rvecs, R, p, delta, 0, R, out_triples, cap, count);
}

// A window of the slot order (multiples of kSlotAlign; the end is clipped to the number of slots): only head rows in
// [h0, h1) and tail rows in [t0, t1) take part.  kgc_join_blocks walks the join window by window.
struct JoinWindow { int64_t h0, h1, t0, t1; };
enum { kPrepFresh = 0,      // grouping, summaries and tail operands are made anew (kgc_join, kgc_join_range)
       kPrepReuse = 1 };    // ... are taken from the handle when they were made for the same join
static int join_range_impl(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                           float delta, int32_t r_begin, int32_t r_end, kgc_triple* out_triples, uint64_t cap, uint64_t* count,
                           const JoinWindow* win, int prep_mode);

int kgc_join_range(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                   float delta, int32_t r_begin, int32_t r_end, kgc_triple* out_triples, uint64_t cap, uint64_t* count) {
  return join_range_impl(hd, E, N, d, Rvecs, R, p, delta, r_begin, r_end, out_triples, cap, count, nullptr, kPrepFresh);
}

static int join_range_impl(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                           float delta, int32_t r_begin, int32_t r_end, kgc_triple* out_triples, uint64_t cap, uint64_t* count,
                           const JoinWindow* win, int prep_mode) {
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
  if (r_begin < 0 || r_end < r_begin || r_end > R) return fail(hd, KGC_E_INVALID, "relation range outside [0, R]");
  const int64_t Rn = (int64_t)r_end - r_begin;          // relations of this call
  if (p != 1 && p != 2) return fail(hd, KGC_E_INVALID, "p must be 1 or 2");
  if (std::isnan(delta)) return fail(hd, KGC_E_INVALID, "delta is NaN");
  if (cap > 0 && !out_triples) return fail(hd, KGC_E_INVALID, "out_triples is NULL with cap > 0");
  if ((uintptr_t)out_triples % 16) return fail(hd, KGC_E_INVALID, "out_triples must be 16-byte aligned");
  hd->err.clear();
  hd->stats = kgc_stats{};
  hd->stats.triples_total = (uint64_t)N * (uint64_t)N * (uint64_t)Rn;
  if (N == 0 || Rn == 0) return KGC_OK;

  hipStream_t st = hd->stream;
  const int dtype = hd->cfg.dtype;
  const bool prune = hd->cfg.prune != KGC_PRUNE_OFF;

  // tile shape
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  const int k16 = (d + kNormCols + 15) / 16;
  // automatic choice.  Dense: the barrier-free head-resident kernel while the head tile fits in LDS with
  // some room to spare (256 rows for KS <= 9, d <= 282; 128 rows for KS <= 19, d <= 602).  Pruned: the head-resident list-walking kernels
  // (KS <= 8, d <= 250; pruned_l2_tile).  Otherwise the streaming kernel.
  // the relation-factorised form (optional, dense L2 only, head tile in LDS) has one tile shape of its own
  const bool fact = hd->cfg.factorised != 0 && p == 2 && !prune && KS <= kDirectMaxKS;
  int tile_id = kDefaultL2Tile;
  if (fact) tile_id = kDirectL2Tile;
  else if (hd->cfg.tile_cfg > 0) tile_id = hd->cfg.tile_cfg - 1;
  else if (!prune && KS <= kDirectMaxKS) tile_id = kDenseL2Tile;
  else if (!prune && KS <= kDirectHalfMaxKS) tile_id = kDirectHalfL2Tile;
  else if (prune) tile_id = pruned_l2_tile(N, KS, kDefaultL2Tile);
  const TileCfg tc = kL2Tiles[tile_id];
  // pruned L2 joins on the 128 x 128 head-resident tiles may go tile by tile instead (decided per batch on the device)
  const bool pairs_ok = prune && p == 2 && tile_id == kResidentL2Tile;
  if (p == 2 && prune && !tc.listed_kernel)
    return fail(hd, KGC_E_INVALID, "this tile variant has no pruned mode; choose a streaming variant");
  const int BM = (p == 2) ? tc.bm : kL1Tile, BN = (p == 2) ? tc.bn : kL1Tile;

  if ((rc = ensure(hd, hd->counters, sizeof(DevCounters))) || (rc = ensure(hd, hd->params, sizeof(JoinParams))))
    return rc;
  DevCounters* cnt = (DevCounters*)hd->counters.p;
  JoinParams* prm = (JoinParams*)hd->params.p;

  // what the handle holds from an earlier call of the same logical join may be taken over
  kgc_handle::Prep& pr = hd->prep;
  const bool reuse = prep_mode != kPrepFresh && pr.valid && pr.E == E && pr.Rv == Rvecs && pr.N == N && pr.d == d && pr.p == p &&
                     pr.dtype == dtype && pr.prune == (int)prune && pr.tile_id == tile_id && pr.delta == delta &&
                     pr.group_radius == hd->cfg.group_radius && !fact;
  KGC_HIP(hd, hipEventRecord(hd->ev[0], st));
  if (!reuse) {
    k_fill_u32<<<grid_for(sizeof(DevCounters) / 4, 256), 256, 0, st>>>((uint32_t*)cnt, sizeof(DevCounters) / 4, 0u);
  } else {    // (the running maxima of the staged tail rows stay)
    k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)cnt, 12, 0u);
    k_fill_u32<<<1, 64, 0, st>>>(&cnt->n_exact, 2, 0u);
  }
  pr.valid = false;

  // ---- row order: identity, or entities grouped around local pivots (pruning) ----
  int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  uint64_t n_groups = 0;
  UnitTable ut{};                 // two-level bound test: filled after the layout
  bool use_units = false;
  bool fine_direct = false;       // ... whose micro-tile level then sums centre distances directly (no M x M matrix)
  if (reuse) {
    Nslots = pr.Nslots; n_groups = pr.n_groups; ut = pr.ut;
  } else if (prune) {
    if ((rc = group_rows(hd, E, N, d, p, delta, KS, k16, &Nslots, &n_groups, &ut)) != KGC_OK) return rc;
  } else {
    if ((rc = ensure(hd, hd->slot_ent, Nslots * 4))) return rc;
    k_identity_slots<<<grid_for(Nslots, 256), 256, 0, st>>>((int32_t*)hd->slot_ent.p, N, Nslots);
  }
  const int32_t* slot_ent = (const int32_t*)hd->slot_ent.p;
  const int nH = (int)(Nslots / BM), nT = (int)(Nslots / BN);
  const int64_t n_micro = Nslots / kMicro;
  const int words_per_row = (nT + 31) / 32;
  const int64_t tiles_per_rel = (int64_t)nH * nT;
  if (nH > 65535) return fail(hd, KGC_E_INVALID, "N too large for one launch grid");

  // ---- relation batches: staged A operands (L2) and the tile lists (pruning) must fit the workspace ----
  const int64_t ws = hd->ws_override > 0 ? hd->ws_override
                                           : hd->cfg.workspace_bytes > 0 ? hd->cfg.workspace_bytes : kDefaultWorkspace;
  const size_t opA_per_rel = (p == 2) ? (size_t)KS * Nslots * kSliceK * 2 : 0;
  int64_t RBmax = Rn;
  if (p == 2 && !fact) RBmax = std::max<int64_t>(1, std::min<int64_t>(Rn, ws / (int64_t)(opA_per_rel + Nslots * 4)));
  if (fact) RBmax = std::max<int64_t>(1, std::min<int64_t>(Rn, ws / (int64_t)(Nslots * 4)));      // u[r][slot]
  if (prune) RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, kMaxTileList / tiles_per_rel));
  RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, 65535));
  if (prune && tiles_per_rel > kMaxTileList) return fail(hd, KGC_E_INVALID, "N too large for the pruned tile list");

  if (p == 2) {
    if ((rc = ensure(hd, hd->opB, (size_t)KS * Nslots * kSliceK * 2)) ||
        (rc = ensure(hd, hd->opA, opA_per_rel * (size_t)(fact ? 1 : RBmax))) || (rc = ensure(hd, hd->normsB, Nslots * 4)) ||
        (rc = ensure(hd, hd->normsA, (size_t)(fact ? 1 : RBmax) * Nslots * 4)))
      return rc;
    if (fact && ((rc = ensure(hd, hd->relu, (size_t)RBmax * Nslots * 4)) || (rc = ensure(hd, hd->reln, RBmax * 4)) ||
                 (rc = ensure(hd, hd->limr, RBmax * 4))))
      return rc;
  }
  if (prune) {
    if ((rc = ensure(hd, hd->cent, (size_t)n_micro * d * 4)) || (rc = ensure(hd, hd->rad, n_micro * 4)) ||
        (rc = ensure(hd, hd->bitmap, (size_t)RBmax * nH * words_per_row * 4)) ||
        (rc = ensure(hd, hd->row_start, (size_t)RBmax * nH * 4)) ||
        (rc = ensure(hd, hd->row_count, (size_t)RBmax * nH * 4)) ||
        (rc = ensure(hd, hd->cols, (size_t)RBmax * tiles_per_rel * 4)) ||
        (pairs_ok && (rc = ensure(hd, hd->tile_rows, (size_t)RBmax * tiles_per_rel * 4))) ||
        (rc = ensure(hd, hd->active_rows, (size_t)RBmax * nH * 4)) || (rc = ensure(hd, hd->cnorm, n_micro * 4)))
      return rc;
    if (p == 2 && ((rc = ensure(hd, hd->gram, (size_t)n_micro * n_micro * 4)) ||
                   (rc = ensure(hd, hd->relu, (size_t)RBmax * n_micro * 4)) || (rc = ensure(hd, hd->reln, RBmax * 4))))
      return rc;
    // the two-level test pays when the units are clearly fewer than the micro-tiles (groups of several micro-tiles)
    use_units = delta >= 0.f && ut.n_units > 0 && ut.n_units < (1 << 24) && (int64_t)ut.n_units * 10 <= n_micro * 6;
    if (use_units && ((rc = ensure(hd, hd->cent_u, (size_t)ut.n_units * d * 4)) || (rc = ensure(hd, hd->rad_u, (size_t)ut.n_units * 4)) ||
                      (rc = ensure(hd, hd->cnorm_u, (size_t)ut.n_units * 4)) ||
                      (rc = ensure(hd, hd->pair_list, kBoundPairCap * 8)) || (rc = ensure(hd, hd->pair_count, 8))))
      return rc;
    // with few micro-tiles the M x M matrix of centre distances and the R x M products cost more than the handful of
    // micro-tile pairs that are looked up in them
    fine_direct = use_units && p == 2 && n_micro <= 8192;
    if (use_units && p == 2 && ((rc = ensure(hd, hd->gram_u, (size_t)ut.n_units * ut.n_units * 4)) ||
                                (rc = ensure(hd, hd->relu_u, (size_t)RBmax * ut.n_units * 4))))
      return rc;
  }
  const int nbatch = (int)((Rn + RBmax - 1) / RBmax);
  const bool timed = !hd->static_mode;          // per-batch event pairs (creating events allocates)
  while (timed && (int)hd->join_ev.size() < 2 * nbatch) {
    hipEvent_t e;
    KGC_HIP(hd, hipEventCreate(&e));
    hd->join_ev.push_back(e);
  }

  RecheckCtx cx;
  cx.E = E; cx.Et = E; cx.Rv = Rvecs; cx.rstride = d; cx.hstride = 0; cx.tstride = 0; cx.slot_ent = slot_ent; cx.slot_ent_t = slot_ent; cx.dtype = dtype; cx.d = d; cx.p = p;
  cx.delta = (double)delta; cx.out = out_triples; cx.cap = cap; cx.no_self = hd->no_self;
  cx.hit_counter = &cnt->hits; cx.cand_counter = &cnt->candidates;
  set_alignment(cx);

  KGC_HIP(hd, hipEventRecord(hd->ev[3], st));     // end of grouping
  if (prune && !reuse) {
    if (p == 2) {
      k_micro_summary<2><<<(unsigned)n_micro, 64, 0, st>>>(E, dtype, d, slot_ent, n_micro, (float*)hd->cent.p,
                                                            (float*)hd->rad.p, (float*)hd->cnorm.p);
      if (!fine_direct) {
        // squared distances between all micro-tile centres, once: the part of the bound that no relation changes
        TileDistArgs ta{};
        ta.X = hd->cent.p; ta.dtypeX = KGC_F32; ta.n_rows = n_micro; ta.Y = hd->cent.p; ta.dtypeY = KGC_F32;
        ta.n_cols = n_micro; ta.shift = nullptr; ta.dtype_shift = KGC_F32; ta.d = d; ta.matrix = (float*)hd->gram.p; ta.symmetric = 1;
        const dim3 g((unsigned)((n_micro + 127) / 128), (unsigned)((n_micro + 127) / 128), 1);
        if (n_micro <= 4096)      // few centres: small tiles, so that the launch fills the chip; the flat test takes its pair terms ready made
          k_small_matrix<2><<<dim3((unsigned)((n_micro + 31) / 32), (unsigned)((n_micro + 31) / 32), 1), 256, 0, st>>>(
              hd->cent.p, KGC_F32, n_micro, (const float*)hd->cent.p, n_micro, d, (float*)hd->gram.p,
              (!use_units && delta >= 0.f) ? (const float*)hd->rad.p : nullptr, delta, 1);
        else
          k_tile_dist<2, kEpiMatrix><<<g, 256, 0, st>>>(ta);
      }
      if (use_units) {
        k_unit_summary<2><<<(unsigned)ut.n_units, 64, 0, st>>>((const float*)hd->cent.p, (const float*)hd->rad.p, d, ut,
                                                            (float*)hd->cent_u.p, (float*)hd->rad_u.p, (float*)hd->cnorm_u.p);
        TileDistArgs tu{};
        tu.X = hd->cent_u.p; tu.dtypeX = KGC_F32; tu.n_rows = ut.n_units; tu.Y = hd->cent_u.p; tu.dtypeY = KGC_F32;
        tu.n_cols = ut.n_units; tu.shift = nullptr; tu.dtype_shift = KGC_F32; tu.d = d; tu.matrix = (float*)hd->gram_u.p; tu.symmetric = 1;
        const dim3 gu((unsigned)((ut.n_units + 127) / 128), (unsigned)((ut.n_units + 127) / 128), 1);
        k_tile_dist<2, kEpiMatrix><<<gu, 256, 0, st>>>(tu);
      }
    } else {
      k_micro_summary<1><<<(unsigned)n_micro, 64, 0, st>>>(E, dtype, d, slot_ent, n_micro, (float*)hd->cent.p,
                                                            (float*)hd->rad.p, (float*)hd->cnorm.p);
      if (use_units)
        k_unit_summary<1><<<(unsigned)ut.n_units, 64, 0, st>>>((const float*)hd->cent.p, (const float*)hd->rad.p, d, ut,
                                                               (float*)hd->cent_u.p, (float*)hd->rad_u.p, (float*)hd->cnorm_u.p);
    }
  }
  const size_t stage_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
  if (reuse) {
    // tail operands, summaries and (L1) the join parameters are in place
  } else if (p == 2) {
    k_stage_operands<false><<<grid_for(Nslots / kStageRows, 1), 256, stage_lds, st>>>(
        E, Rvecs, dtype, d, 0, 1, slot_ent, Nslots, KS, (uint16_t*)hd->opB.p, (float*)hd->normsB.p, cnt->max_b, nullptr, nullptr, 0, kStageRows,
        0, nullptr, fact ? -1.f : delta);      // (the factorised filter has an error analysis of its own: plain norms)
    if (fact)     // the head side of the factorised form carries no relation: the plain rows, once
      k_stage_operands<true><<<grid_for(Nslots / kStageRows, 1), 256, stage_lds, st>>>(
          E, nullptr, dtype, d, 0, 1, slot_ent, Nslots, KS, (uint16_t*)hd->opA.p, (float*)hd->normsA.p, cnt->max_a, nullptr,
          nullptr, 0, kStageRows);
  } else {
    k_row_l1_max<<<grid_for(N * 32, 256), 256, 0, st>>>(E, N, d, dtype, cnt->max_a);
    k_row_l1_max<<<grid_for((int64_t)R * 32, 256), 256, 0, st>>>(Rvecs, R, d, dtype, cnt->max_b);
    k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, 0);
  }
  KGC_HIP(hd, hipEventRecord(hd->ev[1], st));
  const bool bitmap_ready = reuse && pr.bitmap_valid && pr.bm_r0 == r_begin && pr.bm_r1 == r_end && nbatch == 1;
  pr.E = E; pr.Rv = Rvecs; pr.N = N; pr.d = d; pr.p = p; pr.dtype = dtype; pr.prune = (int)prune; pr.tile_id = tile_id;
  pr.delta = delta; pr.group_radius = hd->cfg.group_radius; pr.Nslots = Nslots; pr.n_groups = n_groups; pr.ut = ut;
  pr.bitmap_valid = false;
  // the window in join tiles (whole problem without one)
  int wH0 = 0, wH1 = nH, wT0 = 0, wT1 = nT;
  if (win) {
    wH0 = (int)(std::min(win->h0, Nslots) / BM); wH1 = (int)(std::min(win->h1, Nslots) / BM);
    wT0 = (int)(std::min(win->t0, Nslots) / BN); wT1 = (int)(std::min(win->t1, Nslots) / BN);
    if ((rc = ensure(hd, hd->active_rows, (size_t)RBmax * (Nslots / kSlotAlign) * 4 + 4))) return rc;
  }
  const int nHw = wH1 - wH0, nTw = wT1 - wT0;
  const bool empty_window = nHw <= 0 || nTw <= 0;
  RecheckCtx cxw = cx;               // dense launches over a window count their slots from the window's start
  cxw.slot_ent = slot_ent + (int64_t)wH0 * BM; cxw.slot_ent_t = slot_ent + (int64_t)wT0 * BN;

  int b = 0;
  for (int64_t r0 = r_begin; r0 < r_end && !empty_window; r0 += RBmax, ++b) {
    const int RB = (int)std::min<int64_t>(RBmax, r_end - r0);
    const uint32_t* row_start = nullptr;
    const uint32_t* row_count = nullptr;
    const uint32_t* cols = nullptr;
    const uint32_t* active_rows = nullptr;
    const unsigned int* n_active = nullptr;
    if (prune) {
      // a2: bound test on micro-tile pairs -> bitmap of join tiles -> per-row lists of surviving tail tiles
      const int64_t bm_words = (int64_t)RB * nH * words_per_row;
      if (!bitmap_ready) k_fill_u32<<<grid_for(bm_words, 256), 256, 0, st>>>((uint32_t*)hd->bitmap.p, bm_words, 0u);
      // The bound test (flat, or the micro-tile level of the two-level one) can list the surviving tiles itself; when they are few, that list serves the tile-at-a-time
      // join kernel and the pass over the bitmap is skipped (the device decides, k_batch_tiles).  Not with a window:
      // the list would hold the tiles outside it too.
      const bool direct_lists = pairs_ok && !win && !bitmap_ready && delta >= 0.f && p == 2;
      if (b > 0) k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)&cnt->tile_cursor, 3, 0u);      // cursor and n_active (zero at the start of a call)
      if (bitmap_ready) {
        // the bound test of these relations is still in the bitmap (the previous window of the same relation range)
      } else if (delta >= 0.f && p == 2) {
        // u[rl][m] = r . c_m as a tiled product, ||r||^2 by one wave per relation
        k_rel_centre_dot<<<grid_for((int64_t)RB * 64, 256), 256, 0, st>>>(
            Rvecs, dtype, d, (int)r0, RB, (const float*)hd->cent.p, 0, (float*)hd->relu.p, (float*)hd->reln.p);
        if (!fine_direct) {
          TileDistArgs td{};
          td.X = (const char*)Rvecs + (size_t)r0 * d * (dtype == KGC_BF16 ? 2 : 4); td.dtypeX = dtype; td.n_rows = RB;
          td.Y = hd->cent.p; td.dtypeY = KGC_F32; td.n_cols = n_micro; td.shift = nullptr; td.dtype_shift = KGC_F32;
          td.d = d; td.matrix = (float*)hd->relu.p;
          if (n_micro <= 4096 && RB <= 4096)
            launch_small_dot(st, td.X, dtype, RB, (const float*)hd->cent.p, n_micro, d, (float*)hd->relu.p);
          else
            k_tile_dist<0, kEpiMatrix><<<dim3((unsigned)((n_micro + 127) / 128), (unsigned)((RB + 127) / 128), 1), 256, 0, st>>>(td);
        }
        BoundL2Args ba{};
        ba.D = fine_direct ? nullptr : (const float*)hd->gram.p; ba.u = (const float*)hd->relu.p; ba.rn = (const float*)hd->reln.p;
        ba.cent = (const float*)hd->cent.p; ba.Rv = Rvecs; ba.dtype = dtype; ba.r0 = (int)r0;
        ba.rad = (const float*)hd->rad.p; ba.cnorm = (const float*)hd->cnorm.p; ba.n_micro = n_micro; ba.RB = RB;
        ba.d = d; ba.delta = delta; ba.bitmap = (uint32_t*)hd->bitmap.p; ba.nH = nH; ba.words_per_row = words_per_row;
        ba.micro_per_bm = BM / kMicro; ba.micro_per_bn = BN / kMicro;
        if (direct_lists) {
          ba.list_cols = (uint32_t*)hd->cols.p; ba.list_rows = (uint32_t*)hd->tile_rows.p; ba.list_active = (uint32_t*)hd->active_rows.p;
          ba.list_count = &cnt->tile_cursor;
          ba.list_cap = (unsigned long long)std::min<int64_t>((int64_t)RB * nH, (int64_t)RB * tiles_per_rel);   // what all three arrays hold
        }
        if (use_units) {
          // unit level first (same arithmetic on unit summaries), then the micro-tile pairs of the survivors
          TileDistArgs tu{};
          tu.X = (const char*)Rvecs + (size_t)r0 * d * (dtype == KGC_BF16 ? 2 : 4); tu.dtypeX = dtype; tu.n_rows = RB;
          tu.Y = hd->cent_u.p; tu.dtypeY = KGC_F32; tu.n_cols = ut.n_units; tu.shift = nullptr; tu.dtype_shift = KGC_F32;
          tu.d = d; tu.matrix = (float*)hd->relu_u.p;
          if (ut.n_units <= 8192 && RB <= 4096)      // a thin product: 128 x 128 tiles would leave most of the chip idle
            launch_small_dot(st, tu.X, dtype, RB, (const float*)hd->cent_u.p, ut.n_units, d, (float*)hd->relu_u.p);
          else
            k_tile_dist<0, kEpiMatrix><<<dim3((unsigned)((ut.n_units + 127) / 128), (unsigned)((RB + 127) / 128), 1), 256, 0, st>>>(tu);
          k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)hd->pair_count.p, 2, 0u);
          BoundL2Args bu = ba;
          bu.D = (const float*)hd->gram_u.p; bu.u = (const float*)hd->relu_u.p; bu.rad = (const float*)hd->rad_u.p;
          bu.cnorm = (const float*)hd->cnorm_u.p; bu.n_micro = ut.n_units;
          BoundPairs bp{(unsigned long long*)hd->pair_list.p, (unsigned long long*)hd->pair_count.p, kBoundPairCap};
          if (ut.n_units <= 8192 && (int64_t)ut.n_units * 4 > n_micro) {
            // units of a micro-tile or two (few unit pairs survive): the flat kernel's form -- table, first comparison per
            // chunk, loads in groups -- 137 -> 59 us on the N = 100,000 workload
            const dim3 gu((unsigned)((ut.n_units + 255) / 256), (unsigned)((ut.n_units + kHeadsFlat - 1) / kHeadsFlat),
                          (unsigned)((RB + kRelChunk - 1) / kRelChunk));
            if (direct_lists) k_bound_l2<false, true, true><<<gu, 256, 0, st>>>(bu, ba, ut, bp);
            else k_bound_l2<false, true, false><<<gu, 256, 0, st>>>(bu, ba, ut, bp);
          } else {                       // large units (many pairs survive, the first comparison rarely ends a chunk): the plain form (2.4 against 3.2 ms per batch on the N = 1,000,000 workload)
            const dim3 gu((unsigned)((ut.n_units + 255) / 256), (unsigned)((ut.n_units + kHeadChunk - 1) / kHeadChunk),
                          (unsigned)((RB + kRelChunk - 1) / kRelChunk));
            if (direct_lists) k_bound_l2_units<true><<<gu, 256, 0, st>>>(bu, ba, ut, bp);
            else k_bound_l2_units<false><<<gu, 256, 0, st>>>(bu, ba, ut, bp);
          }
          if (direct_lists) k_bound_refine<true><<<dim3(1024, 32, 1), 256, 0, st>>>(ba, ut, bp);
          else k_bound_refine<false><<<dim3(1024, 32, 1), 256, 0, st>>>(ba, ut, bp);
        } else {
          const dim3 g((unsigned)((n_micro + 255) / 256), (unsigned)((n_micro + kHeadsFlat - 1) / kHeadsFlat),
                       (unsigned)((RB + kRelChunk - 1) / kRelChunk));
          if (n_micro <= 4096) k_bound_l2<true, false><<<g, 256, 0, st>>>(ba, ba, UnitTable{}, BoundPairs{});       // (the matrix came from k_small_matrix with radii)
          else k_bound_l2<false, false><<<g, 256, 0, st>>>(ba, ba, UnitTable{}, BoundPairs{});
        }
      } else if (delta >= 0.f) {
        TileDistArgs ta{};
        ta.X = hd->cent.p; ta.dtypeX = KGC_F32; ta.row_ids = nullptr; ta.n_rows_dev = nullptr; ta.n_rows = n_micro;
        ta.Y = hd->cent.p; ta.dtypeY = KGC_F32; ta.col_ids = nullptr; ta.n_cols_dev = nullptr; ta.n_cols = n_micro;
        ta.shift = Rvecs; ta.dtype_shift = dtype; ta.r0 = (int)r0; ta.d = d;
        ta.rad = (const float*)hd->rad.p; ta.delta = delta; ta.bitmap = (uint32_t*)hd->bitmap.p;
        ta.nH = nH; ta.words_per_row = words_per_row; ta.micro_per_bm = BM / kMicro; ta.micro_per_bn = BN / kMicro;
        if (use_units) {
          // unit level first (unit centres and radii in place of the micro-tile ones), then the micro-tile pairs
          TileDistArgs tu = ta;
          tu.X = hd->cent_u.p; tu.Y = hd->cent_u.p; tu.n_rows = ut.n_units; tu.n_cols = ut.n_units; tu.rad = (const float*)hd->rad_u.p;
          tu.ut = ut; tu.bp = BoundPairs{(unsigned long long*)hd->pair_list.p, (unsigned long long*)hd->pair_count.p, kBoundPairCap};
          tu.fine_cent = (const float*)hd->cent.p; tu.fine_rad = (const float*)hd->rad.p; tu.n_micro = n_micro;
          k_fill_u32<<<1, 64, 0, st>>>((uint32_t*)hd->pair_count.p, 2, 0u);
          const dim3 gu((unsigned)((ut.n_units + 127) / 128), (unsigned)((ut.n_units + 127) / 128), (unsigned)RB);
          k_tile_dist<1, kEpiBoundUnits><<<gu, 256, 0, st>>>(tu);
          k_bound_refine_l1<<<dim3(1024, 32, 1), 256, 0, st>>>(tu);
        } else {
          const dim3 g((unsigned)((n_micro + 127) / 128), (unsigned)((n_micro + 127) / 128), (unsigned)RB);
          k_tile_dist<1, kEpiBound><<<g, 256, 0, st>>>(ta);
        }
      }
      if (direct_lists)
        k_batch_tiles<<<1, 64, 0, st>>>(cnt, 1, 1, (unsigned long long)RB * nH,
                                        (unsigned long long)std::min<int64_t>((int64_t)RB * nH, (int64_t)RB * tiles_per_rel));
      k_rows_from_bitmap<<<(unsigned)(((int64_t)RB * nH + 256 * bitmap_rows_per_lane(words_per_row) - 1) / (256 * bitmap_rows_per_lane(words_per_row))), 256, 0, st>>>(
          (const uint32_t*)hd->bitmap.p, words_per_row, (int64_t)RB * nH, (uint32_t*)hd->row_start.p,
          (uint32_t*)hd->row_count.p, (uint32_t*)hd->cols.p, &cnt->tile_cursor, (uint32_t*)hd->active_rows.p,
          &cnt->n_active, pairs_ok ? (uint32_t*)hd->tile_rows.p : nullptr, nH, wH0, wH1, wT0, wT1,
          direct_lists ? &cnt->pair_mode : nullptr, direct_lists ? &cnt->tiles : nullptr);
      if (!direct_lists) k_batch_tiles<<<1, 64, 0, st>>>(cnt, pairs_ok ? 1 : 0, 0, 0ull, 0ull);
      row_start = (const uint32_t*)hd->row_start.p;
      row_count = (const uint32_t*)hd->row_count.p;
      cols = (const uint32_t*)hd->cols.p;
      active_rows = (const uint32_t*)hd->active_rows.p;
      n_active = &cnt->n_active;
    }
    // pruned launches stride a fixed grid over the active rows (their number is only known on the device)
    const unsigned row_grid = (unsigned)std::min<int64_t>((int64_t)RB * nH, 4096);
    if (fact) {
      // u[rl][slot] = r . e for the batch (tiled float32 product; padding slots stay 0), ||r||^2, thresholds
      k_fill_u32<<<grid_for((int64_t)RB * Nslots, 256), 256, 0, st>>>((uint32_t*)hd->relu.p, (int64_t)RB * Nslots, 0u);
      TileDistArgs td{};
      td.X = (const char*)Rvecs + (size_t)r0 * d * (dtype == KGC_BF16 ? 2 : 4); td.dtypeX = dtype; td.n_rows = RB;
      td.Y = E; td.dtypeY = dtype; td.col_ids = slot_ent; td.n_cols = Nslots; td.shift = nullptr; td.dtype_shift = dtype;
      td.d = d; td.matrix = (float*)hd->relu.p;
      k_tile_dist<0, kEpiMatrix><<<dim3((unsigned)((Nslots + 127) / 128), (unsigned)((RB + 127) / 128), 1), 256, 0, st>>>(td);
      k_rel_centre_dot<<<grid_for((int64_t)RB * 64, 256), 256, 0, st>>>(Rvecs, dtype, d, (int)r0, RB, nullptr, 0,
                                                                     (float*)hd->relu.p, (float*)hd->reln.p);
      k_fact_params<<<grid_for(RB, 256), 256, 0, st>>>(cnt, (const float*)hd->reln.p, RB, delta, dtype, d, KS * kSliceK,
                                                      (float*)hd->limr.p);
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b], st));
      JoinFactArgs fa{};
      fa.A = (const uint16_t*)hd->opA.p; fa.B = (const uint16_t*)hd->opB.p; fa.u = (const float*)hd->relu.p;
      fa.limr = (const float*)hd->limr.p; fa.Nslots = Nslots; fa.KS = KS; fa.k16 = k16; fa.nH = nH; fa.nT = nT;
      fa.r0 = (int)r0; fa.RB = RB; fa.cx = cx;
      const size_t head_bytes = (size_t)KS * 256 * kSliceK * 2;
      fa.rc = (int)std::max<size_t>(1, std::min<size_t>(64, (kMaxLds - head_bytes) / (256 * 4)));
      const size_t dyn_lds = head_bytes + (size_t)fa.rc * 256 * 4;
      // tail tiles in ranges of about 3 MiB of staged rows (they stay in L2 while the head tiles pass), cut
      // further when there are too few head tiles to fill the chip
      const int64_t tile_bytes = (int64_t)BN * KS * kSliceK * 2;
      int64_t nsplit = (nT * tile_bytes + kL2RangeBytesResident - 1) / kL2RangeBytesResident;
      nsplit = std::max<int64_t>(nsplit, (1024 + nH - 1) / nH);
      nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, std::min<int64_t>(nT, 65535)));
      KGC_HIP(hd, hipFuncSetAttribute((const void*)k_join_l2_fact<2, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds));
      hipLaunchKernelGGL((k_join_l2_fact<2, 4>), dim3((unsigned)nH, (unsigned)nsplit, 1), dim3(512), dyn_lds, st, fa);
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b + 1], st));
    } else if (p == 2) {
      int stage_grid = prune ? (int)std::min<int64_t>((int64_t)RB * nH * (BM / kStageRows), 4096)
                             : grid_for((int64_t)RB * (Nslots / kStageRows), 1);
      int stage_nh = nH, stage_bm = BM;
      if (win && !prune) {      // dense join over a window: only its head rows are staged, as a list of 256-row tiles
        const int n256 = (int)(Nslots / kSlotAlign), w0 = (int)((int64_t)wH0 * BM / kSlotAlign), w1 = (int)((int64_t)wH1 * BM / kSlotAlign);
        k_window_rows<<<grid_for((int64_t)RB * (w1 - w0), 256), 256, 0, st>>>((uint32_t*)hd->active_rows.p, &cnt->n_active, RB, n256, w0, w1);
        active_rows = (const uint32_t*)hd->active_rows.p; n_active = &cnt->n_active;
        stage_nh = n256; stage_bm = (int)kSlotAlign;
        stage_grid = (int)std::min<int64_t>((int64_t)RB * (w1 - w0) * (kSlotAlign / kStageRows), 16384);
      }
      k_stage_operands<true><<<stage_grid, 256, stage_lds, st>>>(
          E, Rvecs, dtype, d, (int)r0, RB, slot_ent, Nslots, KS, (uint16_t*)hd->opA.p, (float*)hd->normsA.p,
          cnt->max_a, active_rows, n_active, stage_nh, stage_bm, 0, nullptr, delta);
      if (win && !prune) { active_rows = nullptr; n_active = nullptr; }
      k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, KS * kSliceK);
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b], st));
      if (tc.stream_kernel) {
        JoinStreamArgs sa{};      // the fields a launch does not use stay zero
        sa.A = (const uint16_t*)hd->opA.p; sa.B = (const uint16_t*)hd->opB.p; sa.prm = prm; sa.Nslots = Nslots;
        sa.KS = KS; sa.k16 = k16; sa.nH = nH; sa.nT = nT; sa.r0 = (int)r0; sa.RB = RB;
        sa.row_start = row_start; sa.row_count = row_count; sa.cols = cols; sa.active_rows = active_rows;
        sa.n_active = n_active; sa.cx = cx;
        if (!prune) {      // dense: the window by its first tiles (pruned: the tile lists hold only the window's tiles)
          sa.A += (size_t)wH0 * BM * kSliceK; sa.B += (size_t)wT0 * BN * kSliceK; sa.nH = nHw; sa.nT = nTw; sa.cx = cxw;
        }
        // Dense: tail tiles are cut into ranges of about kL2RangeBytes of staged B rows and the range is the
        // slowest grid dimension, so that a range stays in the 4 MiB L2 of every XCD while all head tiles of
        // all relations of the batch pass over it (the tail rows then cost almost no HBM traffic; what remains
        // is one read of every head tile per range); small problems are cut further to fill the chip.
        // Pruned: one block per row.
        int64_t nsplit = 1;
        if (!prune) {
          const int64_t tile_bytes = (int64_t)BN * KS * kSliceK * 2;
          const int64_t range_bytes = hd->cfg.range_kib > 0 ? (int64_t)hd->cfg.range_kib * 1024
                                      : (tc.head_resident ? resident_range_bytes(nTw * tile_bytes) : kL2RangeBytes);
          nsplit = (nTw * tile_bytes + range_bytes - 1) / range_bytes;
          nsplit = std::max<int64_t>(nsplit, (4096 + (int64_t)nHw * RB - 1) / ((int64_t)nHw * RB));
          nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, std::min<int64_t>(nTw, 65535)));
        }
        void (*kern)(const JoinStreamArgs) = prune ? tc.listed_kernel : tc.stream_kernel;
        if (tile_id == kDenseL2Tile) {
          if (KS > kDirectMaxKS) return fail(hd, KGC_E_INVALID, "d too large for the head-resident tile variant");
          kern = dense_kernel_for(k16);
        }
        size_t dyn_lds = 0;
        if (tc.head_resident) {
          dyn_lds = ((size_t)KS * BM + (size_t)tc.tail_buffers * BN) * kSliceK * 2;
          if ((dyn_lds + tc.static_lds) * tc.blocks_per_cu > kMaxLds) return fail(hd, KGC_E_INVALID, "d too large for the head-resident tile variant");
          if (prune && tc.tail_buffers == 0) {    // the barrier-free form keeps a row's tile list behind the head slices, in segments if need be
            if (dyn_lds + 1024 > kMaxLds) return fail(hd, KGC_E_INVALID, "d too large for the pruned barrier-free tile variant");
            sa.cols_lds = (int)std::min<size_t>((kMaxLds - dyn_lds) / 4, (size_t)nT);
            if (hd->list_seg_cap > 0) sa.cols_lds = std::min(sa.cols_lds, hd->list_seg_cap);
            dyn_lds += (size_t)sa.cols_lds * 4;
          }
          if (prune && tc.tail_buffers > 0) {     // room for a row's tile list behind the tail buffers, if the LDS has it
            const size_t spare = kMaxLds / tc.blocks_per_cu - (dyn_lds + tc.static_lds);
            sa.cols_lds = (int)std::min<size_t>(spare / 4, (size_t)nT);
            if (sa.cols_lds < nT) sa.cols_lds = 0;             // a list may hold every tail tile: all or nothing
            dyn_lds += (size_t)sa.cols_lds * 4;
          }
          KGC_HIP(hd, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds));
        }
        // (the barrier-free kernel deals rows to workgroups in sets of 256: its grid is a whole number of sets)
        const dim3 grid = prune ? dim3(tile_id == kDirectL2Tile ? (row_grid + 255u) & ~255u : row_grid, 1, 1)
                                : dim3((unsigned)nHw, (unsigned)RB, (unsigned)nsplit);
        // the head-resident and streaming kernels list the accumulator blocks that hold candidates; a kernel of its own
        // then scores the list (the barrier-free dense kernels re-score in place: their candidates are few per tile)
        const bool lists_blocks = tile_id != kDenseL2Tile && tile_id != kDirectL2Tile && tile_id != kDirectL2Tile + 1 &&
                                  tile_id != kDirectHalfL2Tile;
        if (lists_blocks) {
          if ((rc = ensure(hd, hd->xlist, (size_t)hd->xcap * sizeof(ExactEntry)))) return rc;
          sa.xlist = (ExactEntry*)hd->xlist.p; sa.xcount = &cnt->n_exact; sa.xcap = hd->xcap;
        }
        if (pairs_ok) { sa.tile_rows = (const uint32_t*)hd->tile_rows.p; sa.tile_total = &cnt->tile_cursor; sa.pair_mode = &cnt->pair_mode; }
        hipLaunchKernelGGL(kern, grid, dim3(tc.threads), dyn_lds, st, sa);
        if (pairs_ok) {          // the same batch tile by tile, when the device chose that (the other kernel then returned at once)
          const size_t pair_lds = (size_t)2 * KS * 128 * kSliceK * 2;
          KGC_HIP(hd, hipFuncSetAttribute((const void*)k_join_l2_pairs, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pair_lds));
          hipLaunchKernelGGL(k_join_l2_pairs, dim3(hd->pairs_grid), dim3(256), pair_lds, st, sa);      // two resident blocks per compute unit, each walks its tiles
        }
        if (lists_blocks) {
          launch_exact_blocks(st, (const ExactEntry*)hd->xlist.p, &cnt->n_exact, hd->xcap, &cnt->exact_total, &cnt->exact_need, sa.cx);
          if (r0 + RBmax < r_end) k_fill_u32<<<1, 64, 0, st>>>(&cnt->n_exact, 1, 0u);      // an empty list for the next batch
        }
      } else {
        JoinArgs ja{};
        ja.A = (const uint16_t*)hd->opA.p + (size_t)wH0 * BM * kSliceK; ja.B = (const uint16_t*)hd->opB.p + (size_t)wT0 * BN * kSliceK; ja.prm = prm;
        ja.Nslots = Nslots; ja.KS = KS; ja.k16 = k16; ja.nH = nHw; ja.nT = nTw; ja.r0 = (int)r0; ja.RB = RB; ja.cx = cxw;
        hipLaunchKernelGGL(tc.tile_kernel, dim3((unsigned)nTw, (unsigned)nHw, (unsigned)RB), dim3(tc.threads), 0, st, ja);
      }
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b + 1], st));
    } else {
      JoinL1Args la{};
      la.prm = prm; la.Nslots = Nslots; la.nH = nH; la.nT = nT; la.r0 = (int)r0; la.RB = RB;
      la.row_start = row_start; la.row_count = row_count; la.cols = cols; la.active_rows = active_rows;
      la.n_active = n_active; la.cx = cx;
      if (!prune) { la.nH = nHw; la.nT = nTw; la.cx = cxw; }
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b], st));
      hipLaunchKernelGGL(k_join_l1, prune ? dim3(row_grid, 1, 1) : dim3((unsigned)nTw, (unsigned)nHw, (unsigned)RB), dim3(256), 0,
                         st, la);
      if (timed) KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b + 1], st));
    }
    hd->stats.join_launches++;
  }
  KGC_HIP(hd, hipGetLastError());
  KGC_HIP(hd, hipMemcpyAsync(hd->host_counters, cnt, 48, hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipEventRecord(hd->ev[2], st));
  KGC_HIP(hd, wait_event(hd->ev[2]));

  pr.valid = !fact;                  // what the handle now holds describes this join
  pr.bitmap_valid = prune && nbatch == 1 && !empty_window; pr.bm_r0 = r_begin; pr.bm_r1 = r_end;
  // A batch that wanted to list more accumulator blocks than the list holds has dropped the rest (and counted
  // them): the list grows to what was asked for and the join runs again from the start.
  if (hd->host_counters->exact_need > hd->xcap) {
    const unsigned long long need = hd->host_counters->exact_need;
    hd->xcap = (unsigned int)std::min<unsigned long long>(need + need / 4 + 1024, 0xffffffffull);
    return join_range_impl(hd, E, N, d, Rvecs, R, p, delta, r_begin, r_end, out_triples, cap, count, win,
                           prep_mode == kPrepFresh ? kPrepReuse : prep_mode);      // (what was just prepared is still good)
  }

  kgc_stats& s = hd->stats;
  s.emitted = hd->host_counters->hits;
  s.candidates = hd->host_counters->candidates;
  s.tiles_total = (uint64_t)tiles_per_rel * (uint64_t)Rn;
  s.tiles_evaluated = prune ? hd->host_counters->tiles : s.tiles_total;
  s.tiles_pruned = s.tiles_total - s.tiles_evaluated;
  s.pairs_evaluated = prune ? s.tiles_evaluated * (uint64_t)BM * (uint64_t)BN : s.triples_total;
  s.groups = n_groups;
  s.tile_m = BM; s.tile_n = BN;
  s.k_padded = (p == 2) ? k16 * 16 : d;
  s.relation_batches = nbatch;
  s.join_variant = (p == 2) ? (fact ? 100 : tile_id + 1) : 0;
  s.exact_blocks = (int32_t)std::min<unsigned long long>(hd->host_counters->exact_total, 2147483647ull);
  // phase times from the events: [ev0 grouping ev3 | summaries + B staging ev1 | per batch: bound test + A staging | join]
  float ms = 0.f, ms_group = 0.f, ms_between = 0.f;
  (void)hipEventElapsedTime(&s.ms_total, hd->ev[0], hd->ev[2]);
  (void)hipEventElapsedTime(&ms_group, hd->ev[0], hd->ev[3]);
  (void)hipEventElapsedTime(&s.ms_precompute, hd->ev[3], hd->ev[1]);
  if (!timed && hipEventElapsedTime(&ms, hd->ev[1], hd->ev[2]) == hipSuccess) s.ms_join = ms;   // staging of the batches included
  for (int i = 0; timed && i < nbatch; ++i) {
    if (hipEventElapsedTime(&ms, hd->join_ev[2 * i], hd->join_ev[2 * i + 1]) == hipSuccess) s.ms_join += ms;
    hipEvent_t prev = i == 0 ? hd->ev[1] : hd->join_ev[2 * i - 1];
    if (hipEventElapsedTime(&ms, prev, hd->join_ev[2 * i]) == hipSuccess) ms_between += ms;
  }
  // the per-batch gap holds the bound test (pruning) and the A staging (precompute); it is booked under pruning
  // when pruning is on, since A staging then only touches surviving head tiles
  s.ms_prune = prune ? ms_group + ms_between : 0.f;
  if (!prune) s.ms_precompute += ms_group + ms_between;

  *count = s.emitted;
  return s.emitted > cap ? KGC_OVERFLOW : KGC_OK;
}


// The join block by block (Section 4.7).  The slot order of the join (the grouped order with pruning on, the entity
// order otherwise) is cut into blocks of block_rows rows, the relations into ranges of rel_block, and the units
// (relation range, head block, tail block) are joined one after the other, in that order, each through the kernels
// of kgc_join over a window.  Grouping, summaries and the staged tail operands are made by the first unit and
// reused by the others, also across calls; the bound test of a relation range is reused by the units of that range.
int kgc_join_blocks(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, int32_t p,
                    float delta, int64_t block_rows, int32_t rel_block, kgc_cursor* cursor, kgc_triple* out_triples,
                    uint64_t cap, uint64_t* count) {
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  if (!cursor) return fail(hd, KGC_E_INVALID, "cursor is NULL");
  if (block_rows < 1 || rel_block < 1) return fail(hd, KGC_E_INVALID, "block_rows and rel_block must be positive");
  if (hd->cfg.factorised) return fail(hd, KGC_E_INVALID, "kgc_join_blocks does not take the relation-factorised form");
  if (hd->static_mode) return fail(hd, KGC_E_INVALID, "kgc_join_blocks allocates: not available inside kgc_join_static");
  cursor->need = 0;
  if (N <= 0 || R <= 0) {            // (negative sizes are reported by the checks of the join itself)
    uint64_t c = 0;
    const int rc0 = join_range_impl(hd, E, N, d, Rvecs, R, p, delta, 0, R < 0 ? 0 : R, out_triples, cap, &c, nullptr, kPrepFresh);
    cursor->unit = 0; cursor->units = 0;
    return rc0;
  }
  const int64_t brows = (block_rows + kSlotAlign - 1) / kSlotAlign * kSlotAlign;      // blocks are whole 256-row tiles
  const bool prune = hd->cfg.prune != KGC_PRUNE_OFF;
  const int64_t n_rel = ((int64_t)R + rel_block - 1) / rel_block;
  if (cursor->unit > 0) {
    // a continued join: the handle must still hold this join's row order (a grouped order cannot be made again the same)
    const kgc_handle::Prep& pr = hd->prep;
    const bool same = pr.valid && pr.E == E && pr.Rv == Rvecs && pr.N == N && pr.d == d && pr.p == p && pr.delta == delta;
    if (prune && !same)
      return fail(hd, KGC_E_INVALID, "the handle no longer holds this join's row order: start again with a zeroed cursor");
  }
  uint64_t written = 0;
  kgc_stats total{};
  for (;;) {
    // blocks per side: known once the row order is (the grouped order pads its groups); the first unit is (0, 0, 0) anyway
    int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
    if (hd->prep.valid && hd->prep.E == E && hd->prep.N == N) Nslots = hd->prep.Nslots;
    else if (cursor->unit > 0 && prune) return fail(hd, KGC_E_INVALID, "the handle lost this join's row order");
    const int64_t nb = (Nslots + brows - 1) / brows;
    const uint64_t units = (uint64_t)n_rel * (uint64_t)nb * (uint64_t)nb;
    cursor->units = units;
    if (cursor->unit >= units) break;
    const uint64_t u = cursor->unit;
    const int64_t rr = (int64_t)(u / (uint64_t)(nb * nb)), bh = (int64_t)((u / (uint64_t)nb) % (uint64_t)nb), bt = (int64_t)(u % (uint64_t)nb);
    const JoinWindow w{bh * brows, (bh + 1) * brows, bt * brows, (bt + 1) * brows};
    const int32_t r_lo = (int32_t)(rr * rel_block), r_hi = (int32_t)std::min<int64_t>((int64_t)R, (rr + 1) * (int64_t)rel_block);
    uint64_t c = 0;
    const int rc = join_range_impl(hd, E, N, d, Rvecs, R, p, delta, r_lo, r_hi, out_triples ? out_triples + written : nullptr,
                                   cap - written, &c, &w, u == 0 ? kPrepFresh : kPrepReuse);
    if (rc != KGC_OK && rc != KGC_OVERFLOW) return rc;
    if (rc == KGC_OVERFLOW) {         // the unit does not fit what is left of the buffer: it stays to be done
      cursor->need = c;
      hd->stats = total; hd->stats.emitted = written;
      *count = written;
      return KGC_OVERFLOW;
    }
    written += c;
    const kgc_stats& b = hd->stats;
    total.triples_total += b.triples_total; total.tiles_total += b.tiles_total; total.tiles_evaluated += b.tiles_evaluated;
    total.tiles_pruned += b.tiles_pruned; total.pairs_evaluated += b.pairs_evaluated; total.candidates += b.candidates;
    total.join_launches += b.join_launches; total.ms_total += b.ms_total; total.ms_precompute += b.ms_precompute;
    total.ms_prune += b.ms_prune; total.ms_join += b.ms_join; total.relation_batches += b.relation_batches;
    total.exact_blocks += b.exact_blocks; total.groups = b.groups; total.tile_m = b.tile_m; total.tile_n = b.tile_n;
    total.k_padded = b.k_padded; total.join_variant = b.join_variant;
    cursor->unit = u + 1;
  }
  hd->stats = total; hd->stats.emitted = written;
  hd->stats.triples_total = (uint64_t)N * (uint64_t)N * (uint64_t)R;
  *count = written;
  return KGC_OK;
}

}  // extern "C"

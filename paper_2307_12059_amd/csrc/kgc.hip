// Host side of the kgc C ABI (see include/kgc.h): argument checks, scratch management, launch order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "kgc_kernels.h"

using namespace kgc;

namespace {

constexpr int kMaxD = 960;                      // keeps kernel 1's LDS tile under 64 KiB
constexpr int64_t kSlotAlign = 256;            // rows are padded to a multiple of the largest tile
constexpr int64_t kDefaultWorkspace = 16ll << 30;
constexpr int64_t kL2RangeBytes = 1ll << 20;
constexpr size_t kMaxLds = 160 * 1024;         // LDS per workgroup on gfx950

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

struct TileCfg {
  int bm, bn, threads;
  void (*tile_kernel)(const JoinArgs);            // one block per tile pair
  void (*stream_kernel)(const JoinStreamArgs);    // one block per (relation, head tile), streaming over tail tiles
  bool head_resident;                             // stream_kernel keeps the head tile's K slices in LDS (dynamic LDS)
};

// Tile variants of kernel 2 (tile_cfg = index + 1).
const TileCfg kL2Tiles[] = {
    {128, 128, 256, k_join_l2<128, 128, 2, 2>, nullptr, false},
    {256, 128, 256, k_join_l2<256, 128, 2, 2>, nullptr, false},
    {256, 256, 256, k_join_l2<256, 256, 2, 2>, nullptr, false},
    {128, 128, 512, k_join_l2<128, 128, 4, 2>, nullptr, false},
    {256, 256, 512, k_join_l2<256, 256, 4, 2>, nullptr, false},
    {256, 256, 256, nullptr, k_join_l2_stream<256, 256, 2, 2, 1>, false},
    {256, 128, 256, nullptr, k_join_l2_stream<256, 128, 2, 2, 2>, false},
    {128, 128, 256, nullptr, k_join_l2_stream<128, 128, 2, 2, 2>, false},
    {256, 256, 512, nullptr, k_join_l2_stream<256, 256, 4, 2, 1>, false},
    {128, 256, 256, nullptr, k_join_l2_stream<128, 256, 2, 2, 2>, false},
    {256, 256, 512, nullptr, k_join_l2_ares<256, 4, 2>, true},
    {256, 256, 512, nullptr, k_join_l2_ares<256, 2, 4>, true},
    {256, 128, 512, nullptr, k_join_l2_ares<128, 4, 2>, true},
};
constexpr int kDefaultL2Tile = 8;                 // index into kL2Tiles
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

int grid_for(int64_t items, int per_block) { return (int)std::min<int64_t>((items + per_block - 1) / per_block, 1 << 20); }

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
  if (!(c.group_radius >= 0.f)) return KGC_E_INVALID;
  for (int v : c.reserved)
    if (v != 0) return KGC_E_INVALID;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return KGC_E_HIP;
  kgc_handle* h = new (std::nothrow) kgc_handle();
  if (!h) return KGC_E_NOMEM;
  h->cfg = c;
  h->stream = (hipStream_t)c.stream;
  if (hipGetDevice(&h->device) != hipSuccess) { delete h; return KGC_E_HIP; }
  if (hipHostMalloc((void**)&h->host_counters, sizeof(DevCounters), hipHostMallocDefault) != hipSuccess) {
    delete h;
    return KGC_E_NOMEM;
  }
  for (auto& e : h->ev)
    if (hipEventCreate(&e) != hipSuccess) { kgc_destroy(h); return KGC_E_HIP; }
  *out = h;
  return KGC_OK;
}

void kgc_destroy(kgc_handle* h) {
  if (!h) return;
  release(h->slot_ent); release(h->opB); release(h->opA); release(h->normsB); release(h->normsA);
  release(h->counters); release(h->params);
  if (h->host_counters) (void)hipHostFree(h->host_counters);
  for (auto& e : h->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : h->join_ev)
    if (e) (void)hipEventDestroy(e);
  delete h;
}

const char* kgc_last_error(const kgc_handle* h) { return h ? h->err.c_str() : "null handle"; }

int kgc_get_stats(const kgc_handle* h, kgc_stats* out) {
  if (!h || !out) return KGC_E_INVALID;
  *out = h->stats;
  return KGC_OK;
}

int kgc_norms(kgc_handle* hd, const void* E, int64_t N, int32_t d, const void* Rvecs, int32_t R, float* nB,
              float* nA) {
  int rc = check_common(hd, E, N, d, Rvecs, R);
  if (rc != KGC_OK) return rc;
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
                                               (uint16_t*)hd->opB.p, (float*)hd->normsB.p, nullptr);
    k_scatter_norms<<<grid_for(Nslots, 256), 256, 0, st>>>((const float*)hd->normsB.p, (const int32_t*)hd->slot_ent.p,
                                                           Nslots, N, 1, nB);
  }
  if (nA) {
    for (int r = 0; r < R; ++r) {
      k_stage_operands<true><<<g, 256, stage_lds, st>>>(E, Rvecs, dtype, d, r, 1, (const int32_t*)hd->slot_ent.p, Nslots, KS,
                                                (uint16_t*)hd->opA.p, (float*)hd->normsB.p, nullptr);
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
  if (!hd) return KGC_E_INVALID;
  if (!count) return fail(hd, KGC_E_INVALID, "count is NULL");
  *count = 0;
  int rc = check_common(hd, E, N, d, Rvecs, R);
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

  // tile shape
  int tile_id = hd->cfg.tile_cfg > 0 ? hd->cfg.tile_cfg - 1 : kDefaultL2Tile;
  const TileCfg tc = kL2Tiles[tile_id];
  const int BM = (p == 2) ? tc.bm : kL1Tile, BN = (p == 2) ? tc.bn : kL1Tile;
  const int64_t Nslots = (N + kSlotAlign - 1) / kSlotAlign * kSlotAlign;
  const int nH = (int)(Nslots / BM), nT = (int)(Nslots / BN);
  const int KS = (d + kNormCols + kSliceK - 1) / kSliceK;
  const int k16 = (d + kNormCols + 15) / 16;

  // relation batches: staged A operands of a batch must fit the workspace, and the grid 2^31 blocks
  const int64_t ws = hd->cfg.workspace_bytes > 0 ? hd->cfg.workspace_bytes : kDefaultWorkspace;
  const size_t opA_per_rel = (p == 2) ? (size_t)KS * Nslots * kSliceK * 2 : 0;
  int64_t RBmax = R;
  if (p == 2) RBmax = std::max<int64_t>(1, std::min<int64_t>(R, ws / (int64_t)(opA_per_rel + Nslots * 4)));
  // dense launches use a (tail tile, head tile, relation) grid; y and z are limited to 65535 blocks
  const int64_t tiles_per_rel = (int64_t)nH * nT;
  RBmax = std::max<int64_t>(1, std::min<int64_t>(RBmax, 65535));
  if (nH > 65535) return fail(hd, KGC_E_INVALID, "N too large for one launch grid");

  if ((rc = ensure(hd, hd->slot_ent, Nslots * 4)) || (rc = ensure(hd, hd->counters, sizeof(DevCounters))) ||
      (rc = ensure(hd, hd->params, sizeof(JoinParams))))
    return rc;
  if (p == 2) {
    if ((rc = ensure(hd, hd->opB, (size_t)KS * Nslots * kSliceK * 2)) ||
        (rc = ensure(hd, hd->opA, opA_per_rel * (size_t)RBmax)) || (rc = ensure(hd, hd->normsB, Nslots * 4)) ||
        (rc = ensure(hd, hd->normsA, (size_t)RBmax * Nslots * 4)))
      return rc;
  }
  const int nbatch = (int)((R + RBmax - 1) / RBmax);
  while ((int)hd->join_ev.size() < 2 * nbatch) {
    hipEvent_t e;
    KGC_HIP(hd, hipEventCreate(&e));
    hd->join_ev.push_back(e);
  }

  DevCounters* cnt = (DevCounters*)hd->counters.p;
  JoinParams* prm = (JoinParams*)hd->params.p;
  const int32_t* slot_ent = (const int32_t*)hd->slot_ent.p;

  KGC_HIP(hd, hipEventRecord(hd->ev[0], st));
  k_fill_u32<<<grid_for(sizeof(DevCounters) / 4, 256), 256, 0, st>>>((uint32_t*)cnt, sizeof(DevCounters) / 4, 0u);
  k_identity_slots<<<grid_for(Nslots, 256), 256, 0, st>>>((int32_t*)hd->slot_ent.p, N, Nslots);

  RecheckCtx cx;
  cx.E = E; cx.Rv = Rvecs; cx.slot_ent = slot_ent; cx.dtype = dtype; cx.d = d; cx.p = p;
  cx.delta = (double)delta; cx.out = out_triples; cx.cap = cap;
  cx.hit_counter = &cnt->hits; cx.cand_counter = &cnt->candidates;

  float ms_pre_extra = 0.f;
  const size_t stage_lds = (size_t)kStageRows * (KS * kSliceK + 8) * 2;
  if (p == 2) {
    k_stage_operands<false><<<grid_for(Nslots / kStageRows, 1), 256, stage_lds, st>>>(
        E, Rvecs, dtype, d, 0, 1, slot_ent, Nslots, KS, (uint16_t*)hd->opB.p, (float*)hd->normsB.p, cnt->max_b);
  } else {
    k_row_l1_max<<<grid_for(N * 32, 256), 256, 0, st>>>(E, N, d, dtype, cnt->max_a);
    k_row_l1_max<<<grid_for((int64_t)R * 32, 256), 256, 0, st>>>(Rvecs, R, d, dtype, cnt->max_b);
    k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, 0);
  }
  KGC_HIP(hd, hipEventRecord(hd->ev[1], st));

  int b = 0;
  for (int64_t r0 = 0; r0 < R; r0 += RBmax, ++b) {
    const int RB = (int)std::min<int64_t>(RBmax, R - r0);
    if (p == 2) {
      k_stage_operands<true><<<grid_for((int64_t)RB * (Nslots / kStageRows), 1), 256, stage_lds, st>>>(
          E, Rvecs, dtype, d, (int)r0, RB, slot_ent, Nslots, KS, (uint16_t*)hd->opA.p, (float*)hd->normsA.p,
          cnt->max_a);
      k_join_params<<<1, 64, 0, st>>>(cnt, prm, delta, p, dtype, d, KS * kSliceK);
      JoinArgs ja;
      ja.A = (const uint16_t*)hd->opA.p; ja.B = (const uint16_t*)hd->opB.p; ja.prm = prm;
      ja.Nslots = Nslots; ja.KS = KS; ja.k16 = k16; ja.nH = nH; ja.nT = nT; ja.r0 = (int)r0; ja.RB = RB;
      ja.worklist = nullptr; ja.cx = cx;
      KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b], st));
      if (tc.stream_kernel) {
        JoinStreamArgs sa;
        sa.A = ja.A; sa.B = ja.B; sa.prm = prm; sa.Nslots = Nslots; sa.KS = KS; sa.k16 = k16; sa.nH = nH; sa.nT = nT;
        sa.r0 = (int)r0; sa.RB = RB; sa.row_ptr = nullptr; sa.row_key = nullptr; sa.cols = nullptr; sa.cx = cx;
        // Tail tiles are cut into ranges of about kL2RangeBytes of staged B rows, so that the blocks running at
        // the same time (consecutive head tiles of one range) keep their B rows in the 4 MiB L2 of their XCD;
        // small problems are cut further to fill the chip.
        const int64_t tile_bytes = (int64_t)BN * KS * kSliceK * 2;
        int64_t nsplit = (nT * tile_bytes + kL2RangeBytes - 1) / kL2RangeBytes;
        nsplit = std::max<int64_t>(nsplit, (4096 + (int64_t)nH * RB - 1) / ((int64_t)nH * RB));
        nsplit = std::max<int64_t>(1, std::min<int64_t>(nsplit, std::min<int64_t>(nT, 65535)));
        size_t dyn_lds = 0;
        if (tc.head_resident) {
          dyn_lds = ((size_t)KS * 256 + 2 * (size_t)BN) * kSliceK * 2;
          if (dyn_lds > kMaxLds) return fail(hd, KGC_E_INVALID, "d too large for the head-resident tile variant");
          KGC_HIP(hd, hipFuncSetAttribute((const void*)tc.stream_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)dyn_lds));
        }
        hipLaunchKernelGGL(tc.stream_kernel, dim3((unsigned)nH, (unsigned)nsplit, (unsigned)RB), dim3(tc.threads), dyn_lds,
                           st, sa);
      } else {
        hipLaunchKernelGGL(tc.tile_kernel, dim3((unsigned)nT, (unsigned)nH, (unsigned)RB), dim3(tc.threads), 0, st, ja);
      }
      KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b + 1], st));
    } else {
      JoinL1Args la;
      la.prm = prm; la.Nslots = Nslots; la.nH = nH; la.nT = nT; la.r0 = (int)r0; la.RB = RB;
      la.worklist = nullptr; la.cx = cx;
      KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b], st));
      hipLaunchKernelGGL(k_join_l1, dim3((unsigned)nT, (unsigned)nH, (unsigned)RB), dim3(256), 0, st, la);
      KGC_HIP(hd, hipEventRecord(hd->join_ev[2 * b + 1], st));
    }
    hd->stats.join_launches++;
  }
  KGC_HIP(hd, hipGetLastError());
  KGC_HIP(hd, hipMemcpyAsync(hd->host_counters, cnt, 16, hipMemcpyDeviceToHost, st));
  KGC_HIP(hd, hipEventRecord(hd->ev[2], st));
  KGC_HIP(hd, hipStreamSynchronize(st));

  kgc_stats& s = hd->stats;
  s.emitted = hd->host_counters->hits;
  s.candidates = hd->host_counters->candidates;
  s.tiles_total = (uint64_t)tiles_per_rel * (uint64_t)R;
  s.tiles_evaluated = s.tiles_total;
  s.tiles_pruned = 0;
  s.pairs_evaluated = s.triples_total;
  s.tile_m = BM; s.tile_n = BN;
  s.k_padded = (p == 2) ? k16 * 16 : d;
  s.relation_batches = nbatch;
  float ms = 0.f;
  (void)hipEventElapsedTime(&s.ms_total, hd->ev[0], hd->ev[2]);
  (void)hipEventElapsedTime(&s.ms_precompute, hd->ev[0], hd->ev[1]);
  for (int i = 0; i < nbatch; ++i) {
    if (hipEventElapsedTime(&ms, hd->join_ev[2 * i], hd->join_ev[2 * i + 1]) == hipSuccess) s.ms_join += ms;
    if (i > 0 && hipEventElapsedTime(&ms, hd->join_ev[2 * i - 1], hd->join_ev[2 * i]) == hipSuccess) ms_pre_extra += ms;
  }
  if (nbatch > 0 && hipEventElapsedTime(&ms, hd->ev[1], hd->join_ev[0]) == hipSuccess) ms_pre_extra += ms;
  s.ms_precompute += ms_pre_extra;
  s.ms_prune = 0.f;

  *count = s.emitted;
  return s.emitted > cap ? KGC_OVERFLOW : KGC_OK;
}

}  // extern "C"

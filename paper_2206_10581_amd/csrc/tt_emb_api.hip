// C ABI of libtt_emb.so: argument checks, workspace carving, launch sequences, timing slots.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "tt_emb_internal.h"

namespace ttemb {

// launchers defined next to their kernels
void launch_sort_pass(const Plan&, const Workspace&, const IdSource& src, int B, int pass, hipStream_t,
                      int which);
void launch_seg_count(const Plan&, const Workspace&, int B, hipStream_t);
void launch_seg_write(const Plan&, const Workspace&, int B, hipStream_t);
void launch_group(const Plan&, const Workspace&, int B, hipStream_t, int which);
void launch_prefix_fwd(const Plan&, const Workspace&, const float* g1, const float* g2, int B,
                       hipStream_t);
void launch_row_fwd(const Plan&, const Workspace&, const float* g3, int B, float* out, hipStream_t);
void launch_gsum(const Plan&, const Workspace&, const float* grad, int B, hipStream_t);
void launch_gsum_fix(const Plan&, const Workspace&, int B, hipStream_t);
void launch_u_bwd(const Plan&, const Workspace&, const float* g3, const float* grad, int B,
                  hipStream_t);
void launch_dg3(const Plan&, const Workspace&, const float* grad, int B, hipStream_t);
void launch_prefix_bwd(const Plan&, const Workspace&, const float* g1, const float* g2, int B,
                       hipStream_t);
void launch_sgd(const Plan&, const Workspace&, float* g1, float* g2, float* g3, float lr,
                const UpdateRule&, hipEvent_t stop, hipStream_t);
// matrix-core variants for the shapes mfma_shape() accepts
bool mfma_shape(const Shape&);
void launch_prefix_fwd_mfma(const Plan&, const Workspace&, const float* g1, const float* g2, int B,
                            hipStream_t);
void launch_row_fwd_mfma(const Plan&, const Workspace&, const float* g3, int B, float* out,
                         hipStream_t);
void launch_id_bwd_mfma(const Plan&, const Workspace&, const float* g3, const float* grad, int B,
                        hipStream_t);
void launch_prefix_bwd_mfma(const Plan&, const Workspace&, const float* g1, const float* g2, int B,
                            hipStream_t);
bool mfma_fused_mid(const Shape&);
bool gsum_block_rows(const Shape&);
void launch_bwd_mid_mfma(const Plan&, const Workspace&, const float* g1, const float* g2,
                         const float* g3, const float* grad, int B, hipStream_t);
void launch_gsum_block(const Plan&, const Workspace&, const float* grad, int B, hipStream_t);
hipError_t calibrate(void* buf, size_t bytes, hipStream_t, double* copy_bytes_per_s,
                     double* mfma_flops_per_s, double* gather_bytes_per_s,
                     double* far_gather_bytes_per_s);

static const char* const kSlotNames[kSlotCount] = {
    "sort_hist", "sort_scan", "sort_scatter", "seg_count", "seg_write",  "group",
    "prefix_fwd", "row_fwd",  "gsum",         "gsum_fix",  "u_bwd",      "dg3",        "prefix_bwd",
    "sgd",        "event_pair"};

static thread_local std::string g_hip_error = "HIP call failed";

static inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }

static int bits_for(uint32_t v) {  // number of bits needed to write v (at least 1)
  int b = 1;
  while ((v >> b) != 0 && b < 32) ++b;
  return b;
}

static int make_plan(const tt_emb_config* c, Plan* pl) {
  if (c == nullptr) return TT_EMB_EINVAL;
  for (int k = 0; k < 3; ++k)
    if (c->n[k] <= 0 || c->d[k] <= 0 || c->n[k] >= (int64_t(1) << 31) || c->d[k] > 4096)
      return TT_EMB_EINVAL;
  if (c->r[0] <= 0 || c->r[1] <= 0 || c->r[0] > 4096 || c->r[1] > 4096) return TT_EMB_EINVAL;
  if (c->max_batch < 1 || c->max_batch >= (int64_t(1) << 30)) return TT_EMB_EINVAL;
  int64_t n12 = c->n[0] * c->n[1];
  if (n12 >= (int64_t(1) << 31)) return TT_EMB_EINVAL;
  int64_t N = n12 * c->n[2];
  if (N >= (int64_t(1) << 31)) return TT_EMB_EINVAL;
  pl->split = 1;
  pl->user_maxB = c->max_batch;
  pl->user_N = N;
  if (c->n[1] > kMaxBins || c->n[2] > kMaxBins) return TT_EMB_EINVAL;
  int64_t D = (int64_t)c->d[0] * c->d[1] * c->d[2];
  if (D > 4096) return TT_EMB_EINVAL;
  pl->user_D = (int)D;
  const int64_t S2 = (int64_t)c->r[0] * c->d[1] * c->r[1];
  const int64_t PN = (int64_t)c->d[0] * c->d[1] * c->r[1];
  if (S2 > (1 << 24) || PN > (1 << 24)) return TT_EMB_EINVAL;

  // slab split: d1 = 8, 12, ... with everything else fit for the matrix-core kernels, and the
  // enlarged table and batch still inside the 31-bit key and index ranges
  int64_t n1 = c->n[0], maxB = c->max_batch;
  int d1 = c->d[0];
  if (!(c->flags & TT_EMB_FLAG_GENERIC_KERNELS) && d1 > 4 && d1 % 4 == 0 && d1 <= 32) {
    const int k = d1 / 4;
    Shape t{};
    t.d1 = 4;
    t.d2 = c->d[1];
    t.d3 = c->d[2];
    t.r1 = c->r[0];
    t.r2 = c->r[1];
    if (mfma_shape(t) && N * k < (int64_t(1) << 31) && maxB * k < (int64_t(1) << 30)) {
      pl->split = k;
      n1 *= k;
      n12 *= k;
      N *= k;
      maxB *= k;
      D /= k;
      d1 = 4;
    }
  }
  Shape& s = pl->sh;
  s.n1 = (uint32_t)n1;
  s.n2 = (uint32_t)c->n[1];
  s.n3 = (uint32_t)c->n[2];
  s.N = (uint32_t)N;
  s.d1 = d1;
  s.d2 = c->d[1];
  s.d3 = c->d[2];
  s.r1 = c->r[0];
  s.r2 = c->r[1];
  s.M = s.d1 * s.d2;
  s.W = s.d2 * s.r2;
  s.PN = s.d1 * s.W;
  s.D = (int)D;
  s.S1 = s.d1 * s.r1;
  s.S2 = s.r1 * s.W;
  s.S3 = s.r2 * s.d3;

  pl->mfma = mfma_shape(s) && !(c->flags & TT_EMB_FLAG_GENERIC_KERNELS);
  pl->maxB = maxB;
  pl->maxQ = std::min<int64_t>(maxB, n12);
  pl->sortBlocksMax = (int)cdiv64(pl->maxB, kSortItems);
  pl->segBlocksMax = (int)cdiv64(pl->maxB, kSegItems);
  pl->uBlocksMax = (int)cdiv64(pl->maxB, kSortItems);
  pl->qBlocksMax = (int)cdiv64(pl->maxQ, kSortItems);
  pl->tilesMax = (int)cdiv64(pl->maxB, kTileSlots);
  pl->maxChunk3 = cdiv64(pl->maxB, kChunk3Min) + s.n3;
  pl->maxChunk2 = cdiv64(pl->maxQ, kChunk2) + s.n2;
  pl->keyBits = bits_for(s.N);  // the sentinel N itself must be representable
  pl->passes = (pl->keyBits + 10) / 11;
  pl->bitsPerPass = (pl->keyBits + pl->passes - 1) / pl->passes;
  return TT_EMB_OK;
}

// Index sets: one serves the forward/backward pair in flight, two hold the batches prepared ahead,
// and the one that has been idle longest is the next to be filled (a pipeline started two steps
// early has two steps to finish and need not wait for the step that has just ended).
constexpr int kSets = 4;
// The index pipelines run on kSideStreams streams of the library's own, set s on stream
// s % kSideStreams.  Two measure best: with one, a pipeline cannot start before the previous one has
// ended (+11 us per step at config 3); with four, the process has more streams than hardware
// queues (+0.5 us, +1.5 us when the host runs far ahead).
constexpr int kSideStreams = 2;

// Walks the workspace layout; with base == nullptr only the size is computed.  The index arrays
// exist `sets` times (ws[sets..kSets) repeat set 0); the arithmetic buffers are shared.  With
// lookup_only the buffers that only the backward pass uses are left out (their pointers are null).
static size_t carve(const Plan& pl, char* base, Workspace* ws /* [kSets] or nullptr */,
                    int sets = kSets, bool lookup_only = false) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> char* {
    char* p = base ? base + off : nullptr;
    off += (bytes + 255) & ~size_t(255);
    return p;
  };
  const Shape& s = pl.sh;
  const size_t mB = (size_t)pl.maxB, mQ = (size_t)pl.maxQ;
  Workspace set[kSets];
  for (int i = 0; i < sets; ++i) {
    Workspace& w = set[i];
    w.has_order = false;
    w.ctr = (Counters*)take(sizeof(Counters));
    for (int k = 0; k < 2; ++k) w.key[k] = (uint32_t*)take(mB * 4);
    for (int k = 0; k < 2; ++k) w.val[k] = (uint32_t*)take(mB * 4);
    w.cnt = (uint32_t*)take((size_t)pl.sortBlocksMax * kMaxBins * 4);
    w.tot = (uint32_t*)take((size_t)kMaxBins * 4);
    w.seg_nu = (uint32_t*)take((size_t)pl.segBlocksMax * 4);
    w.seg_nq = (uint32_t*)take((size_t)pl.segBlocksMax * 4);
    w.s_u = (int*)take(mB * 4);
    w.s_rec = (int4*)take(mB * 16);
    w.u_rs = (int*)take((mB + 1) * 4);
    w.u_i3 = (int*)take(mB * 4);
    w.u_q = (int*)take(mB * 4);
    w.u_code = (int*)take(mB * 4);
    w.q_us = (int*)take((mQ + 1) * 4);
    w.q_i1 = (int*)take(mQ * 4);
    w.q_i2 = (int*)take(mQ * 4);
    w.cnt3 = (uint32_t*)take((size_t)pl.uBlocksMax * s.n3 * 4);
    w.cnt2 = (uint32_t*)take((size_t)pl.qBlocksMax * s.n2 * 4);
    w.g3_list = (int*)take(mB * 4);
    w.g3_start = (int*)take(((size_t)s.n3 + 1) * 4);
    w.c3_start = (int*)take(((size_t)s.n3 + 1) * 4);
    w.c3_desc = (int4*)take((size_t)pl.maxChunk3 * 16);
    w.c3_item = (int2*)take((size_t)pl.maxChunk3 * kChunk3 * 8);
    w.c3_order = (int*)take((size_t)pl.maxChunk3 * 4);
    w.g2_list = (int*)take(mQ * 4);
    w.g2_start = (int*)take(((size_t)s.n2 + 1) * 4);
    w.c2_start = (int*)take(((size_t)s.n2 + 1) * 4);
    w.c2_desc = (int4*)take((size_t)pl.maxChunk2 * 16);
    w.c2_item = (int4*)take((size_t)pl.maxChunk2 * kChunk2 * 16);
    // g1_first[n1], g1_end[n1], band_cnt, band_cur: one stretch, cleared by the first sort pass
    w.g1_first = (int*)take((size_t)s.n1 * 8 + 2 * kOrderBands * 4);
    w.g1_end = w.g1_first + s.n1;
    w.band_cnt = (uint32_t*)(w.g1_end + s.n1);
    w.band_cur = w.band_cnt + kOrderBands;
  }
  Workspace& w = set[0];
  w.P = (float*)take(mQ * s.PN * 4);
  w.Pt = w.gsum = w.carry = w.dPsum = w.dg1part = w.part3 = w.part2 = nullptr;
  if (!lookup_only) {
    if (pl.mfma && s.r1 >= 64) w.Pt = (float*)take(mQ * s.PN * 4);  // ranks with the two-launch backward
    w.gsum = (float*)take(mB * s.D * 4);
    w.carry = (float*)take((size_t)pl.tilesMax * 2 * s.D * 4);
    w.dPsum = (float*)take(mQ * s.PN * 4);
    w.dg1part = (float*)take(mQ * s.S1 * 4);
    w.part3 = (float*)take((size_t)pl.maxChunk3 * s.S3 * 4);
    w.part2 = (float*)take((size_t)pl.maxChunk2 * s.S2 * 4);
  }
  for (int i = sets; i < kSets; ++i) set[i] = set[0];
  for (int i = 1; i < sets; ++i) {
    set[i].P = w.P;
    set[i].Pt = w.Pt;
    set[i].gsum = w.gsum;
    set[i].carry = w.carry;
    set[i].dPsum = w.dPsum;
    set[i].dg1part = w.dg1part;
    set[i].part3 = w.part3;
    set[i].part2 = w.part2;
  }
  if (ws)
    for (int i = 0; i < kSets; ++i) ws[i] = set[i];
  return off;
}

struct EventPair {
  int slot;
  hipEvent_t a, b;
};

}  // namespace ttemb

using namespace ttemb;

struct tt_emb {
  tt_emb_config cfg;
  Plan plan;
  Workspace ws[kSets];  // index sets over shared arithmetic buffers
  int cur;            // set of the latest forward (and of the backward that follows it)
  float *g1, *g2, *g3;
  const int32_t* reindex;  // old id -> table row applied in front of the split, or nullptr
  UpdateRule ada;          // kind kUpdateSgd: plain SGD
  int64_t adam_step;       // Adam: updates made since tt_emb_set_adam
  int64_t reindex_n;
  int64_t pending_B;  // -1: no forward pending
  int64_t last_B;     // batch size of the latest forward
  bool have_forward;
  hipStream_t last_stream;
  // tt_emb_prepare: index pipelines of coming batches on a stream of the library's own
  hipStream_t side[kSets];  // stream of each index set (kSideStreams distinct ones), created on
                            // first use, default priority
  hipEvent_t ev_fork;   // recorded on the caller's stream, awaited by side
  hipEvent_t done[kSets];   // recorded on the caller's stream after the last kernel that reads the set
  bool done_valid[kSets];   // done[s] covers the latest use of set s
  int recent[kSets];        // index sets of the latest backward_update calls, newest first (-1: none)
  struct Prepared {
    bool valid;         // this index set holds a batch that no forward has consumed yet
    const int64_t* ids;
    int64_t B;
    uint64_t seq;       // order of the prepare calls
    hipEvent_t ready;   // recorded on side when the set is complete
  } prep[kSets];
  uint64_t prep_seq;
  bool profiling;
  bool mfma;  // matrix-core kernels apply to this shape and are not switched off
  std::vector<EventPair> events;
  int64_t prof_launches[kSlotCount];
  double prof_ms[kSlotCount];
};

static IdSource id_source(const tt_emb* h, const int64_t* ids, int64_t base, bool reindexed) {
  const Plan& pl = h->plan;
  return IdSource{ids, base, reindexed ? h->reindex : nullptr, reindexed ? h->reindex_n : 0,
                  pl.split, pl.user_N, (int64_t)pl.sh.n2 * pl.sh.n3};
}

static int hip_fail(hipError_t e) {
  g_hip_error = std::string("HIP: ") + hipGetErrorString(e);
  return TT_EMB_EHIP;
}

// Runs one launcher; with profiling on, brackets it with events on the same stream.
template <class F>
static int run_slot(tt_emb* h, int slot, hipStream_t st, F&& f) {
  EventPair ev{slot, nullptr, nullptr};
  if (h->profiling) {
    hipError_t e = hipEventCreate(&ev.a);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventCreate(&ev.b);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventRecord(ev.a, st);
    if (e != hipSuccess) return hip_fail(e);
  }
  f();
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e);
  if (h->profiling) {
    e = hipEventRecord(ev.b, st);
    if (e != hipSuccess) return hip_fail(e);
    h->events.push_back(ev);
  }
  return TT_EMB_OK;
}

static int drain_events(tt_emb* h) {
  int rc = TT_EMB_OK;
  for (EventPair& ev : h->events) {
    hipError_t e = hipEventSynchronize(ev.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    if (e == hipSuccess) {
      h->prof_ms[ev.slot] += ms;
      h->prof_launches[ev.slot] += 1;
    } else {
      rc = hip_fail(e);
    }
    (void)hipEventDestroy(ev.a);
    (void)hipEventDestroy(ev.b);
  }
  h->events.clear();
  return rc;
}

// Host-side state of a fresh handle (no workspace yet).
static void init_handle(tt_emb* h, const tt_emb_config* cfg, const Plan& pl, float* g1, float* g2,
                        float* g3) {
  h->cfg = *cfg;
  h->plan = pl;
  h->cur = 0;
  for (int i = 0; i < kSets; ++i) h->side[i] = nullptr;
  h->ev_fork = nullptr;
  for (int i = 0; i < kSets; ++i) {
    h->done[i] = nullptr;
    h->done_valid[i] = false;
  }
  h->prep_seq = 0;
  for (int i = 0; i < kSets; ++i) h->recent[i] = -1;
  for (int i = 0; i < kSets; ++i) h->prep[i] = tt_emb::Prepared{false, nullptr, 0, 0, nullptr};
  h->g1 = g1;
  h->g2 = g2;
  h->g3 = g3;
  h->reindex = nullptr;
  h->reindex_n = 0;
  h->ada = UpdateRule{};
  h->adam_step = 0;
  h->pending_B = -1;
  h->last_B = 0;
  h->have_forward = false;
  h->last_stream = nullptr;
  h->profiling = false;
  h->mfma = pl.mfma;
  std::memset(h->prof_launches, 0, sizeof(h->prof_launches));
  std::memset(h->prof_ms, 0, sizeof(h->prof_ms));
}

extern "C" {

int tt_emb_workspace_bytes(const tt_emb_config* cfg, size_t* bytes) {
  Plan pl;
  int rc = make_plan(cfg, &pl);
  if (rc != TT_EMB_OK) return rc;
  if (bytes == nullptr) return TT_EMB_EINVAL;
  *bytes = carve(pl, nullptr, nullptr);
  return TT_EMB_OK;
}

int tt_emb_create(tt_emb_t* out, const tt_emb_config* cfg, float* g1, float* g2, float* g3,
                  void* workspace, size_t workspace_bytes) {
  if (out == nullptr || g1 == nullptr || g2 == nullptr || g3 == nullptr || workspace == nullptr)
    return TT_EMB_EINVAL;
  Plan pl;
  int rc = make_plan(cfg, &pl);
  if (rc != TT_EMB_OK) return rc;
  if (((uintptr_t)workspace & 255u) != 0) return TT_EMB_EINVAL;
  if ((((uintptr_t)g1 | (uintptr_t)g2 | (uintptr_t)g3) & 15u) != 0) return TT_EMB_EINVAL;
  if (workspace_bytes < carve(pl, nullptr, nullptr)) return TT_EMB_ENOSPC;
  tt_emb* h = new (std::nothrow) tt_emb();
  if (h == nullptr) return TT_EMB_EINVAL;
  init_handle(h, cfg, pl, g1, g2, g3);
  carve(pl, (char*)workspace, h->ws);
  *out = h;
  return TT_EMB_OK;
}

// True while st is being captured into a graph.
static bool stream_is_capturing(hipStream_t st) {
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return cap != hipStreamCaptureStatusNone;
}

// Streams and events of tt_emb_prepare, created on its first call: all of them or none (a failure
// half way leaves the handle as it was).
static int setup_side_streams(tt_emb* h) {
  hipStream_t side[kSideStreams] = {};
  hipEvent_t ready[kSets] = {}, done[kSets] = {}, fork = nullptr;
  hipError_t e = hipSuccess;
  for (int i = 0; i < kSideStreams && e == hipSuccess; ++i)
    e = hipStreamCreateWithFlags(&side[i], hipStreamNonBlocking);
  for (int i = 0; i < kSets && e == hipSuccess; ++i) {
    e = hipEventCreateWithFlags(&ready[i], hipEventDisableTiming);
    // the extended launch of the update kernel records kernel times into this one
    if (e == hipSuccess) e = hipEventCreate(&done[i]);
  }
  if (e == hipSuccess) e = hipEventCreateWithFlags(&fork, hipEventDisableTiming);
  if (e != hipSuccess) {
    for (int i = 0; i < kSideStreams; ++i)
      if (side[i] != nullptr) (void)hipStreamDestroy(side[i]);
    for (int i = 0; i < kSets; ++i) {
      if (ready[i] != nullptr) (void)hipEventDestroy(ready[i]);
      if (done[i] != nullptr) (void)hipEventDestroy(done[i]);
    }
    if (fork != nullptr) (void)hipEventDestroy(fork);
    return hip_fail(e);
  }
  for (int i = 0; i < kSets; ++i) {
    h->side[i] = side[i % kSideStreams];
    h->prep[i].ready = ready[i];
    h->done[i] = done[i];
  }
  h->ev_fork = fork;
  return TT_EMB_OK;
}

// Index pipeline of one batch into index set `set`, on stream st.
// how: 0 = everything, including the prefix-ordered schedule of the by-i3 chunks (worth its launch
// only where the pipeline runs beside other work, as in tt_emb_prepare); 1 = no schedule; 2 = a
// lookup: the structures that only the backward pass reads (unique ids by i3) are not built either.
static int run_index(tt_emb* h, int set, const IdSource& src, int B, hipStream_t st, int how) {
  const Plan& pl = h->plan;
  const Workspace& ws = h->ws[set];
  int rc;
  for (int pass = 0; pass < pl.passes; ++pass) {
    rc = run_slot(h, kSlotSortHist, st, [&] { launch_sort_pass(pl, ws, src, B, pass, st, 0); });
    if (rc) return rc;
    if (cdiv64(B, kSortItems) > kFoldScanBlocks) {
      rc = run_slot(h, kSlotSortScan, st, [&] { launch_sort_pass(pl, ws, src, B, pass, st, 2); });
      if (rc) return rc;
    }
    rc = run_slot(h, kSlotSortScatter, st, [&] { launch_sort_pass(pl, ws, src, B, pass, st, 1); });
    if (rc) return rc;
  }
  rc = run_slot(h, kSlotSegCount, st, [&] { launch_seg_count(pl, ws, B, st); });
  if (rc) return rc;
  rc = run_slot(h, kSlotSegWrite, st, [&] { launch_seg_write(pl, ws, B, st); });
  if (rc) return rc;
  h->ws[set].has_order = how == 0;
  return run_slot(h, kSlotGroup, st, [&] { launch_group(pl, ws, B, st, how); });
}

int tt_emb_prepare(tt_emb_t h, const int64_t* ids, int64_t B64, void* hip_stream) {
  if (h == nullptr || B64 < 0) return TT_EMB_EINVAL;
  if (B64 > h->plan.user_maxB) return TT_EMB_ENOSPC;
  if (B64 == 0) return TT_EMB_OK;  // nothing to prepare; forward handles the empty batch itself
  if (ids == nullptr || ((uintptr_t)ids & 7u) != 0) return TT_EMB_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e;
  if (stream_is_capturing(st)) return TT_EMB_ESTATE;  // side streams cannot join a capture
  if (h->side[0] == nullptr) {
    int rc0 = setup_side_streams(h);
    if (rc0) return rc0;
  }
  // Pick the index set to fill.  A set is free when no backward_update still has to be enqueued for
  // it (that is only `cur`, between a forward and its backward) and no prepared batch waits in it.
  // With all taken, the oldest prepared batch is overwritten.
  const bool cur_busy = h->pending_B >= 0;
  int target = -1;
  for (int k = 1; k <= kSets && target < 0; ++k) {
    const int s = (h->cur + k) % kSets;
    if (!h->prep[s].valid && !(s == h->cur && cur_busy)) target = s;
  }
  if (target < 0) {
    for (int s = 0; s < kSets; ++s)
      if (!(s == h->cur && cur_busy) && (target < 0 || h->prep[s].seq < h->prep[target].seq))
        target = s;
  }
  h->prep[target].valid = false;
  // everything that used this set earlier (its backward_update, or an index pipeline that is now
  // dropped) is ordered before: the set's stream is in order, and the fork event covers hip_stream
  if ((h->cfg.flags & TT_EMB_FLAG_IDS_READY) && h->done_valid[target]) {
    // the ids are in memory already: only the set's own last use has to be over
    e = hipStreamWaitEvent(h->side[target], h->done[target], 0);
    if (e != hipSuccess) return hip_fail(e);
  } else {
    e = hipEventRecord(h->ev_fork, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamWaitEvent(h->side[target], h->ev_fork, 0);
    if (e != hipSuccess) return hip_fail(e);
  }
  int rc = run_index(h, target, id_source(h, ids, 0, true), (int)(B64 * h->plan.split),
                     h->side[target], 0);
  if (rc) return rc;
  e = hipEventRecord(h->prep[target].ready, h->side[target]);
  if (e != hipSuccess) return hip_fail(e);
  h->prep[target].valid = true;
  h->prep[target].ids = ids;
  h->prep[target].B = B64;
  h->prep[target].seq = ++h->prep_seq;
  return TT_EMB_OK;
}

}  // extern "C"

// Records that everything that reads index set cur has been enqueued on st (only once
// tt_emb_prepare is in use with TT_EMB_FLAG_IDS_READY: that is who waits for it).
static int mark_set_done(tt_emb* h, hipStream_t st) {
  if (h->done[h->cur] == nullptr || !(h->cfg.flags & TT_EMB_FLAG_IDS_READY)) return TT_EMB_OK;
  hipError_t e = hipEventRecord(h->done[h->cur], st);
  if (e != hipSuccess) return hip_fail(e);
  h->done_valid[h->cur] = true;
  return TT_EMB_OK;
}

// Forward of one batch whose ids come from src (a device array, or consecutive table rows).  With
// arm set the batch stays pending for backward_update.
static int forward_impl(tt_emb* h, const IdSource& src, int64_t B64, float* out, hipStream_t st,
                        bool arm) {
  const int64_t* ids = src.ids;
  h->last_stream = st;
  if (B64 == 0) {
    h->pending_B = arm ? 0 : -1;
    h->have_forward = false;
    return TT_EMB_OK;
  }
  // the matrix-core kernels store rows with 8- and 16-byte accesses; the any-shape kernels store
  // float by float
  if (out == nullptr || ((uintptr_t)out & (h->mfma ? 15u : 3u)) != 0) return TT_EMB_EINVAL;
  const Plan& pl = h->plan;
  // A handle that has used tt_emb_prepare orders its index sets through events on streams of its
  // own, which a capture cannot contain: such a handle is not captured (use a second handle).
  const bool capturing = stream_is_capturing(st);
  if (capturing && h->side[0] != nullptr) return TT_EMB_ESTATE;
  const int B = (int)(B64 * pl.split);  // items of the index pipeline, rows of D/split floats
  h->pending_B = -1;
  int rc;
  // oldest prepared batch with these ids and this size, if any
  int found = -1;
  for (int s = 0; s < kSets; ++s)
    if (ids != nullptr && h->prep[s].valid && h->prep[s].ids == ids && h->prep[s].B == B64 &&
        (found < 0 || h->prep[s].seq < h->prep[found].seq))
      found = s;
  if (found >= 0) {
    // A pipeline that has already finished needs no wait on the caller's stream (its kernels
    // have completed, their results are visible to every later launch); one that has not is
    // awaited on the device.
    const bool finished = hipEventQuery(h->prep[found].ready) == hipSuccess;
    (void)hipGetLastError();  // "not ready" is an answer, not an error
    hipError_t e = finished ? hipSuccess : hipStreamWaitEvent(st, h->prep[found].ready, 0);
    if (e != hipSuccess) return hip_fail(e);
    h->prep[found].valid = false;
    h->cur = found;
  } else {
    // build the index structures here; take a set no prepared batch waits in, else drop one
    int target = -1;
    for (int k = 0; k < kSets && target < 0; ++k)
      if (!h->prep[(h->cur + k) % kSets].valid) target = (h->cur + k) % kSets;
    if (target < 0) {  // every set holds a prepared batch: the oldest one is dropped
      target = 0;
      for (int s = 1; s < kSets; ++s)
        if (h->prep[s].seq < h->prep[target].seq) target = s;
      hipError_t e = hipStreamWaitEvent(st, h->prep[target].ready, 0);
      if (e != hipSuccess) return hip_fail(e);
      h->prep[target].valid = false;
    } else if (h->side[target] != nullptr) {
      // an index pipeline that was dropped earlier may still be writing this set on its stream
      hipError_t e = hipEventRecord(h->ev_fork, h->side[target]);
      if (e != hipSuccess) return hip_fail(e);
      e = hipStreamWaitEvent(st, h->ev_fork, 0);
      if (e != hipSuccess) return hip_fail(e);
    }
    h->cur = target;
    rc = run_index(h, h->cur, src, B, st, arm ? 1 : 2);
    if (rc) return rc;
  }
  h->done_valid[h->cur] = false;  // a new use of this set begins
  const Workspace& ws = h->ws[h->cur];
  rc = run_slot(h, kSlotPrefixFwd, st, [&] {
    if (h->mfma) launch_prefix_fwd_mfma(pl, ws, h->g1, h->g2, B, st);
    else launch_prefix_fwd(pl, ws, h->g1, h->g2, B, st);
  });
  if (rc) return rc;
  rc = run_slot(h, kSlotRowFwd, st, [&] {
    if (h->mfma) launch_row_fwd_mfma(pl, ws, h->g3, B, out, st);
    else launch_row_fwd(pl, ws, h->g3, B, out, st);
  });
  if (rc) return rc;
  h->pending_B = arm ? B : -1;
  h->last_B = B;
  h->have_forward = true;
  if (!arm) return mark_set_done(h, st);  // no backward will follow: the set's use ends here
  return TT_EMB_OK;
}

extern "C" {

int tt_emb_forward(tt_emb_t h, const int64_t* ids, int64_t B64, float* out, void* hip_stream) {
  if (h == nullptr || B64 < 0) return TT_EMB_EINVAL;
  if (B64 > h->plan.user_maxB) return TT_EMB_ENOSPC;
  if (B64 > 0 && (ids == nullptr || ((uintptr_t)ids & 7u) != 0)) return TT_EMB_EINVAL;
  return forward_impl(h, id_source(h, ids, 0, true), B64, out,
                      (hipStream_t)hip_stream, true);
}

int tt_emb_forward_eval(tt_emb_t h, const int64_t* ids, int64_t B64, float* out, void* hip_stream) {
  if (h == nullptr || B64 < 0) return TT_EMB_EINVAL;
  if (B64 > h->plan.user_maxB) return TT_EMB_ENOSPC;
  if (B64 > 0 && (ids == nullptr || ((uintptr_t)ids & 7u) != 0)) return TT_EMB_EINVAL;
  if (h->pending_B >= 0) return TT_EMB_ESTATE;  // would overwrite what the pending backward needs
  return forward_impl(h, id_source(h, ids, 0, true), B64, out,
                      (hipStream_t)hip_stream, false);
}

int tt_emb_materialize(tt_emb_t h, int64_t first_row, int64_t count, float* out, void* hip_stream) {
  if (h == nullptr || first_row < 0 || count < 0) return TT_EMB_EINVAL;
  if (first_row + count > h->plan.user_N) return TT_EMB_EINVAL;
  if (count > 0 && (out == nullptr || ((uintptr_t)out & (h->mfma ? 15u : 3u)) != 0))
    return TT_EMB_EINVAL;
  if (h->pending_B >= 0) return TT_EMB_ESTATE;  // would overwrite what the pending backward needs
  // (every piece starts a multiple of max_batch rows into out: the matrix-core shapes have rows of
  // a multiple of 16 bytes, so the pieces are aligned like out itself)
  const int64_t D = h->plan.user_D;
  for (int64_t off = 0; off < count; off += h->plan.user_maxB) {
    const int64_t nb = std::min<int64_t>(h->plan.user_maxB, count - off);
    int rc = forward_impl(h, id_source(h, nullptr, first_row + off, false), nb, out + off * D,
                          (hipStream_t)hip_stream, false);
    if (rc) return rc;
  }
  return TT_EMB_OK;
}

// ---------------------------------------------------------------------------------------------
// Lookup for callers that cannot allocate: the workspace of the lookup-only forward (one index set
// and the prefix products) lives in a file-scope device array instead of a caller's buffer.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kStaticMaxDevices = 64;
// device address of `scratch` on each device, looked up once per device (every device holds its
// own copy of the array at its own address; the host-side name is never passed to a kernel)
static void* g_scratch_ptr[kStaticMaxDevices];
static std::mutex g_scratch_mutex;

int tt_emb_lookup_static(const tt_emb_config* cfg, const float* g1, const float* g2,
                         const float* g3, const int64_t* ids, int64_t B64, float* out,
                         void* hip_stream) {
  if (cfg == nullptr || g1 == nullptr || g2 == nullptr || g3 == nullptr || B64 < 0)
    return TT_EMB_EINVAL;
  if ((((uintptr_t)g1 | (uintptr_t)g2 | (uintptr_t)g3) & 15u) != 0) return TT_EMB_EINVAL;
  if (B64 > cfg->max_batch) return TT_EMB_ENOSPC;
  if (B64 > 0 && (ids == nullptr || ((uintptr_t)ids & 7u) != 0)) return TT_EMB_EINVAL;
  // the plan, and with it the scratch need, is made for this batch, not for max_batch
  tt_emb_config c = *cfg;
  c.max_batch = B64 > 0 ? B64 : 1;
  Plan pl;
  int rc = make_plan(&c, &pl);
  if (rc != TT_EMB_OK) return rc;
  if (carve(pl, nullptr, nullptr, 1, true) > kStaticScratchBytes) return TT_EMB_ENOSPC;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev != cfg->device || dev < 0 || dev >= kStaticMaxDevices) return TT_EMB_EINVAL;
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
      void* ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess || ptr == nullptr) return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol);
      g_scratch_ptr[dev] = ptr;
    }
    base = g_scratch_ptr[dev];
  }
  if (B64 == 0) return TT_EMB_OK;
  tt_emb h;  // host bookkeeping only, lives for this call
  init_handle(&h, &c, pl, const_cast<float*>(g1), const_cast<float*>(g2), const_cast<float*>(g3));
  carve(pl, (char*)base, h.ws, 1, true);
  return forward_impl(&h, id_source(&h, ids, 0, true), B64, out, (hipStream_t)hip_stream, false);
}

int tt_emb_set_adagrad(tt_emb_t h, float* s1, float* s2, float* s3, float eps) {
  if (h == nullptr) return TT_EMB_EINVAL;
  const bool none = s1 == nullptr && s2 == nullptr && s3 == nullptr;
  if (!none && (s1 == nullptr || s2 == nullptr || s3 == nullptr)) return TT_EMB_EINVAL;
  if ((((uintptr_t)s1 | (uintptr_t)s2 | (uintptr_t)s3) & 15u) != 0) return TT_EMB_EINVAL;
  if (!none && !(eps > 0.f)) return TT_EMB_EINVAL;
  h->ada = UpdateRule{};
  if (!none) {
    h->ada.kind = kUpdateAdagrad;
    h->ada.s1 = s1;
    h->ada.s2 = s2;
    h->ada.s3 = s3;
    h->ada.eps = eps;
  }
  return TT_EMB_OK;
}

int tt_emb_set_adam(tt_emb_t h, float* m1, float* m2, float* m3, float* v1, float* v2, float* v3,
                    float beta1, float beta2, float eps, int64_t steps_done) {
  if (h == nullptr) return TT_EMB_EINVAL;
  float* p[6] = {m1, m2, m3, v1, v2, v3};
  int nulls = 0;
  uintptr_t bits = 0;
  for (float* q : p) {
    nulls += q == nullptr;
    bits |= (uintptr_t)q;
  }
  if ((nulls != 0 && nulls != 6) || (bits & 15u) != 0) return TT_EMB_EINVAL;
  h->ada = UpdateRule{};
  h->adam_step = 0;
  if (nulls == 6) return TT_EMB_OK;
  if (!(eps > 0.f) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) ||
      steps_done < 0)
    return TT_EMB_EINVAL;
  h->ada.kind = kUpdateAdam;
  h->ada.s1 = m1;
  h->ada.s2 = m2;
  h->ada.s3 = m3;
  h->ada.v1 = v1;
  h->ada.v2 = v2;
  h->ada.v3 = v3;
  h->ada.eps = eps;
  h->ada.beta1 = beta1;
  h->ada.beta2 = beta2;
  h->adam_step = steps_done;
  return TT_EMB_OK;
}

int tt_emb_set_reindex(tt_emb_t h, const int32_t* new_id_of, int64_t n_ids) {
  if (h == nullptr || n_ids < 0 || (new_id_of == nullptr && n_ids != 0)) return TT_EMB_EINVAL;
  if (new_id_of != nullptr && ((uintptr_t)new_id_of & 3u) != 0) return TT_EMB_EINVAL;
  if (h->pending_B >= 0) return TT_EMB_ESTATE;  // between a forward and its backward_update
  h->reindex = new_id_of;
  h->reindex_n = new_id_of != nullptr ? n_ids : 0;
  for (int i = 0; i < kSets; ++i) h->prep[i].valid = false;  // prepared batches used the old table
  return TT_EMB_OK;
}

int tt_emb_backward_update(tt_emb_t h, const float* grad_out, float lr, void* hip_stream) {
  if (h == nullptr) return TT_EMB_EINVAL;
  if (h->pending_B < 0) return TT_EMB_ESTATE;
  const int B = (int)h->pending_B;
  // arguments are checked before any state changes: a rejected call leaves the forward pending
  if (B > 0 && (grad_out == nullptr || ((uintptr_t)grad_out & (h->mfma ? 15u : 3u)) != 0))
    return TT_EMB_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  if (B > 0 && h->side[0] != nullptr && stream_is_capturing(st)) return TT_EMB_ESTATE;
  h->pending_B = -1;
  if (B == 0) return TT_EMB_OK;
  const Plan& pl = h->plan;
  const Workspace& ws = h->ws[h->cur];
  int rc;
  // rows of up to 256 floats are summed in blocks of kEntrySlots slots, which no entry crosses;
  // longer rows tile by tile, with a second kernel that joins the runs that cross tiles
  const bool block_sums = h->mfma || gsum_block_rows(pl.sh);
  rc = run_slot(h, kSlotGsum, st, [&] {
    if (block_sums) launch_gsum_block(pl, ws, grad_out, B, st);
    else launch_gsum(pl, ws, grad_out, B, st);
  });
  if (rc) return rc;
  if (!block_sums) {
    rc = run_slot(h, kSlotGsumFix, st, [&] { launch_gsum_fix(pl, ws, B, st); });
    if (rc) return rc;
  }
  if (h->mfma && mfma_fused_mid(pl.sh)) {
    // ranks up to 32: per-id and per-prefix gradient steps in one launch
    rc = run_slot(h, kSlotUBwd, st,
                  [&] { launch_bwd_mid_mfma(pl, ws, h->g1, h->g2, h->g3, grad_out, B, st); });
    if (rc) return rc;
  } else {
    if (h->mfma) {
      rc = run_slot(h, kSlotUBwd, st, [&] { launch_id_bwd_mfma(pl, ws, h->g3, grad_out, B, st); });
      if (rc) return rc;
    } else {
      rc = run_slot(h, kSlotUBwd, st, [&] { launch_u_bwd(pl, ws, h->g3, grad_out, B, st); });
      if (rc) return rc;
      rc = run_slot(h, kSlotDg3, st, [&] { launch_dg3(pl, ws, grad_out, B, st); });
      if (rc) return rc;
    }
    rc = run_slot(h, kSlotPrefixBwd, st, [&] {
      if (h->mfma) launch_prefix_bwd_mfma(pl, ws, h->g1, h->g2, B, st);
      else launch_prefix_bwd(pl, ws, h->g1, h->g2, B, st);
    });
    if (rc) return rc;
  }
  // The update kernel is the last reader of the index set.  Outside stream capture and profiling
  // its completion signal doubles as the set's "done" event.
  // (a handle with side streams is never captured, see forward_impl)
  hipEvent_t stop = nullptr;
  if (h->done[h->cur] != nullptr && (h->cfg.flags & TT_EMB_FLAG_IDS_READY) && !h->profiling)
    stop = h->done[h->cur];
  if (h->ada.kind == kUpdateAdam) {
    // bias corrections of step t = 1, 2, ... (every backward_update with a batch counts)
    const double t = (double)(h->adam_step + 1);
    h->ada.corr1 = (float)(1.0 / (1.0 - std::pow((double)h->ada.beta1, t)));
    h->ada.corr2 = (float)(1.0 / (1.0 - std::pow((double)h->ada.beta2, t)));
  }
  rc = run_slot(h, kSlotSgd, st,
                [&] { launch_sgd(pl, ws, h->g1, h->g2, h->g3, lr, h->ada, stop, st); });
  if (rc) return rc;
  if (h->ada.kind == kUpdateAdam) ++h->adam_step;  // the step counts once its update is enqueued
  if (h->profiling) rc = run_slot(h, kSlotEventPair, st, [] {});
  if (rc) return rc;
  for (int i = kSets - 1; i > 0; --i) h->recent[i] = h->recent[i - 1];
  h->recent[0] = h->cur;
  if (stop != nullptr) {
    h->done_valid[h->cur] = true;
    return TT_EMB_OK;
  }
  return mark_set_done(h, st);
}

int tt_emb_wait_backward(tt_emb_t h, int age) {
  if (h == nullptr || age < 0) return TT_EMB_EINVAL;
  if (age >= kSets - 1) return TT_EMB_OK;  // that set may have been taken again: nothing to wait for
  const int set = h->recent[age];
  if (set < 0 || h->done[set] == nullptr || !h->done_valid[set]) return TT_EMB_OK;
  // the set must not have served a later backward_update (its event would be that later one's)
  for (int i = 0; i < age; ++i)
    if (h->recent[i] == set) return TT_EMB_OK;
  const hipError_t e = hipEventSynchronize(h->done[set]);
  return e == hipSuccess ? TT_EMB_OK : hip_fail(e);
}

int tt_emb_get_stats(tt_emb_t h, int64_t* U, int64_t* Q, int64_t* out_of_range) {
  if (h == nullptr) return TT_EMB_EINVAL;
  Counters c;
  std::memset(&c, 0, sizeof(c));
  int64_t oob = 0;
  if (h->have_forward) {
    hipError_t e = hipStreamSynchronize(h->last_stream);
    if (e != hipSuccess) return hip_fail(e);
    e = hipMemcpy(&c, h->ws[h->cur].ctr, sizeof(c), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e);
    oob = h->last_B - (int64_t)c.nvalid;
  }
  // with a slab split every id, prefix and position was counted once per slab
  const int k = h->plan.split;
  oob /= k;
  if (U) *U = (c.U - c.n_split) / k;
  if (Q) *Q = c.Q / k;
  if (out_of_range) *out_of_range = oob;
  if (c.err != 0) return TT_EMB_EINTERNAL;
  if ((h->cfg.flags & TT_EMB_FLAG_CHECK_RANGE) && oob > 0) return TT_EMB_ERANGE;
  return TT_EMB_OK;
}

int tt_emb_profile_enable(tt_emb_t h, int enable) {
  if (h == nullptr) return TT_EMB_EINVAL;
  int rc = drain_events(h);
  h->profiling = enable != 0;
  std::memset(h->prof_launches, 0, sizeof(h->prof_launches));
  std::memset(h->prof_ms, 0, sizeof(h->prof_ms));
  return rc;
}

int tt_emb_profile_slots(void) { return kSlotCount; }

int tt_emb_profile_read(tt_emb_t h, int slot, const char** name, int64_t* launches, double* ms) {
  if (h == nullptr || slot < 0 || slot >= kSlotCount) return TT_EMB_EINVAL;
  int rc = drain_events(h);
  if (name) *name = kSlotNames[slot];
  if (launches) *launches = h->prof_launches[slot];
  if (ms) *ms = h->prof_ms[slot];
  h->prof_launches[slot] = 0;
  h->prof_ms[slot] = 0.0;
  return rc;
}


int tt_emb_profile_peaks(void* device_buf, size_t bytes, void* hip_stream, double* copy_bytes_per_s,
                         double* mfma_flops_per_s, double* gather_bytes_per_s,
                         double* far_gather_bytes_per_s) {
  if (device_buf == nullptr || copy_bytes_per_s == nullptr || mfma_flops_per_s == nullptr ||
      gather_bytes_per_s == nullptr || far_gather_bytes_per_s == nullptr)
    return TT_EMB_EINVAL;
  if (((uintptr_t)device_buf & 255u) != 0 || bytes < ((size_t)8 << 20)) return TT_EMB_EINVAL;
  const hipError_t e = calibrate(device_buf, bytes, (hipStream_t)hip_stream, copy_bytes_per_s,
                                 mfma_flops_per_s, gather_bytes_per_s, far_gather_bytes_per_s);
  return e == hipSuccess ? TT_EMB_OK : hip_fail(e);
}

int tt_emb_destroy(tt_emb_t h) {
  if (h == nullptr) return TT_EMB_EINVAL;
  (void)drain_events(h);
  if (h->side[0] != nullptr) {
    for (int i = 0; i < kSets; ++i) {
      if (h->side[i] == nullptr) continue;
      (void)hipStreamSynchronize(h->side[i]);
      if (h->prep[i].ready != nullptr) (void)hipEventDestroy(h->prep[i].ready);
      if (h->done[i] != nullptr) (void)hipEventDestroy(h->done[i]);
    }
    for (int i = 0; i < kSideStreams; ++i)
      if (h->side[i] != nullptr) (void)hipStreamDestroy(h->side[i]);
    if (h->ev_fork != nullptr) (void)hipEventDestroy(h->ev_fork);
  }
  delete h;
  return TT_EMB_OK;
}

const char* tt_emb_strerror(int code) {
  switch (code) {
    case TT_EMB_OK: return "ok";
    case TT_EMB_EINVAL: return "invalid argument (null pointer, non-positive or unsupported size)";
    case TT_EMB_ENOSPC: return "batch larger than max_batch, or workspace too small";
    case TT_EMB_ESTATE: return "the handle's state does not allow this call (no pending forward, a pending forward, or a capture on a handle that has prepared)";
    case TT_EMB_EHIP: return g_hip_error.c_str();
    case TT_EMB_ERANGE: return "an id of the last batch was outside [0, N)";
    case TT_EMB_EINTERNAL: return "internal error: a kernel met an impossible index";
    default: return "unknown error code";
  }
}

}  // extern "C"

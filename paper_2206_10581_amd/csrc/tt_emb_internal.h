// Internal declarations shared by the translation units of libtt_emb.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tt_emb.h"

namespace ttemb {

constexpr int kWave = 64;

// stable counting-sort blocks: 16 wavefronts, each owning 256 consecutive items of the block
constexpr int kSortThreads = 1024;
constexpr int kSortWaves = 16;
constexpr int kSortWaveItems = 256;
constexpr int kSortItems = kSortWaves * kSortWaveItems;  // 4096 items per block
constexpr int kFoldRows = 16;       // histogram rows a thread keeps in flight while it adds up a column
constexpr int kFoldScanBlocks = 16;  // sort passes with at most this many blocks need no column-scan launch
constexpr int kMaxBins = 2048;                            // digit / bucket count limit per pass

// The unit of the gradient sums: a run of equal ids is cut at every multiple of kEntrySlots sorted
// slots, and each piece ("entry") is carried through the backward pass like an id of its own - all
// gradient steps are linear in the row gradient, so the pieces of an id simply add up in the same
// matrix-core accumulations that add up the ids of a prefix or of an i3 group.  A block of the
// gradient-sum kernel owns kEntrySlots slots, so no sum ever crosses a block.
constexpr int kEntrySlots = 1024;

constexpr int kSegThreads = 256;
constexpr int kSegItems = 1024;  // sorted slots per block in the segment kernels (4 per thread)

constexpr int kTileSlots = 32;   // sorted slots per wavefront tile in the row kernels
constexpr int kChunk3 = 16;       // record slots per partial sum (chunk) of a G3 slice gradient
// Batches of up to kSmallBatch rows are cut finer where that puts more wavefronts in flight: by-i3
// chunks of 8 ids instead of 16 (-3.7 us per step at 200,000 rows, +6..18 us at 500,000), row tiles
// of 16 slots instead of 32.
constexpr int kSmallBatch = 1 << 18;
constexpr int kChunk3Min = 8;
inline int chunk3_fill(int64_t B) { return B <= kSmallBatch ? kChunk3Min : kChunk3; }
constexpr int kChunk2 = 16;      // unique prefixes per partial sum of a G2 slice gradient
constexpr int kOrderBands = 1024;  // bands of the prefix range the by-i3 chunks are ordered by

// Where the ids of a batch come from, passed to the first sort pass by value.
struct IdSource {
  const int64_t* ids;      // device [B]; nullptr: the consecutive ids base, base+1, ...
  int64_t base;
  const int32_t* reindex;  // device [n_ids] old id -> table row, or nullptr (ids are table rows)
  int64_t n_ids;
  // Slab split (see Plan::split): item idx of the pipeline is slab idx % split of batch position
  // idx / split; rows is the caller's table size N and n23 = n2*n3.
  int split;
  int64_t rows, n23;
};

// Update rule of the update kernel and its caller-owned state (arrays shaped like the cores).
enum UpdateKind { kUpdateSgd = 0, kUpdateAdagrad = 1, kUpdateAdam = 2 };
struct UpdateRule {
  int kind;
  float *s1, *s2, *s3;  // Adagrad: running sums of squared gradients; Adam: first moments
  float *v1, *v2, *v3;  // Adam: second moments
  float eps;
  float beta1, beta2;   // Adam decay rates
  float corr1, corr2;   // Adam bias corrections 1/(1 - beta1^t), 1/(1 - beta2^t) of this step
};

// Table and slice geometry, passed to kernels by value.
struct Shape {
  uint32_t n1, n2, n3, N;  // node factors and N = n1*n2*n3
  int d1, d2, d3, r1, r2;
  int M;   // d1*d2       rows of the partial product
  int W;   // d2*r2       columns of the unfolded G2 slice
  int PN;  // d1*d2*r2    floats of one prefix product
  int D;   // d1*d2*d3    floats of one embedding row
  int S1;  // d1*r1       floats of one G1 slice
  int S2;  // r1*d2*r2    floats of one G2 slice
  int S3;  // r2*d3       floats of one G3 slice
};

// Device-side counters of the latest forward (first bytes of the workspace).
struct Counters {
  int U;        // entries: distinct in-range ids, long runs counted once per kEntrySlots piece
  int Q;        // distinct (i1,i2) prefixes
  int nvalid;   // in-range batch positions (they occupy sorted slots [0, nvalid))
  int nchunk3;  // partial-sum chunks over the by-i3 grouping of unique ids
  int nchunk2;  // partial-sum chunks over the by-i2 grouping of unique prefixes
  int err;      // nonzero: a kernel met an impossible index (bit mask of sites)
  int n_split;  // entries beyond the first of their id (U - n_split distinct ids)
};

// All device arrays carved out of the caller's workspace.
struct Workspace {
  Counters* ctr;
  uint32_t* key[2];   // radix-sort ping-pong keys      [maxB]
  uint32_t* val[2];   // radix-sort ping-pong positions [maxB]
  uint32_t* cnt;      // per-block digit histograms     [sortBlocks * kMaxBins]
  uint32_t* tot;      // digit totals of the current pass  [kMaxBins]
  uint32_t* seg_nu;   // new-id flags per segment block     [segBlocks]
  uint32_t* seg_nq;   // new-prefix flags per segment block [segBlocks]
  int* s_u;           // sorted slot -> unique-id index (-1 for out-of-range ids) [maxB]
  int4* s_rec;        // sorted slot -> {unique-id index, batch position, prefix, i3} [maxB]
  int* u_rs;          // unique id -> first sorted slot  [maxB+1]
  int* u_i3;          // unique id -> i3                 [maxB]
  int* u_q;           // unique id -> prefix index       [maxB]
  int* u_code;        // unique id -> where its gradient row is: batch position, or -(u+1) [maxB]
  int* q_us;          // prefix -> first unique id       [maxQ+1]
  int* q_i1;          // prefix -> i1                    [maxQ]
  int* q_i2;          // prefix -> i2                    [maxQ]
  uint32_t* cnt3;     // per-block histograms of i3 over unique ids   [uBlocks * n3]
  uint32_t* cnt2;     // per-block histograms of i2 over prefixes     [qBlocks * n2]
  int* g3_list;       // unique ids grouped by i3 (stable)  [maxB]
  int* g3_start;      // [n3+1]
  int* c3_start;      // first chunk of each i3 group [n3+1]
  int4* c3_desc;      // chunk -> {i3, first list item, items, 0}  [maxChunk3]
  int2* c3_item;      // chunk, t -> {gradient-row code, prefix} of its t-th id [maxChunk3][kChunk3]
  int* c3_order;      // by-i3 chunks in the order of the prefix of their first id [maxChunk3]
  bool has_order;     // host side: the batch in this set has had c3_order written
  int* g2_list;       // prefixes grouped by i2 (stable) [maxQ]
  int* g2_start;      // [n2+1]
  int* c2_start;      // [n2+1]
  int4* c2_desc;      // chunk -> {i2, first list item, items, 0}  [maxChunk2]
  int4* c2_item;      // chunk, t -> {q, i1, first unique id, end} of its t-th prefix [maxChunk2][kChunk2]
  int* g1_first;      // i1 -> first prefix with that i1 (prefixes are sorted by i1) [n1]
  int* g1_end;        // i1 -> one past its last prefix; directly follows g1_first  [n1]
  uint32_t* band_cnt;  // by-i3 chunks per band of their first prefix; directly follows g1_end
  uint32_t* band_cur;  // chunks placed so far per band; directly follows band_cnt [kOrderBands]
  float* P;           // prefix products G1[i1] G2[i2]   [maxQ][PN]
  float* Pt;          // the same products in the layout the G3-gradient step reads: [maxQ][d2][r2][d1]
                      // (matrix-core shapes of rank 64 and 128 with a backward pass only, else null)
  float* gsum;        // per unique id, sum of its rows' gradients [maxB][D]
  float* carry;       // per tile: head and tail partial sums [tiles][2][D]
  float* dPsum;       // per prefix: gradient of its product  [maxQ][PN]
  float* dg1part;     // per prefix: its term of dG1[i1]      [maxQ][S1]
  float* part3;       // per chunk: partial dG3 slice         [maxChunk3][S3]
  float* part2;       // per chunk: partial dG2 slice         [maxChunk2][S2]
};

struct Plan {
  // Slab split: with d1 = 4*split (split > 1) and the other factors fit for the matrix-core
  // kernels, G1[i1] (d1 x r1) is read as split slices of 4 x r1, i.e. as a table with split*n1
  // first-core slices and d1 = 4 whose row for (split*i1 + h, i2, i3) is the h-th run of D/split
  // floats of the caller's row for (i1, i2, i3).  A batch of B ids is then a batch of split*B ids
  // of that table, out/grad [B][D] are its [split*B][D/split] arrays, and the cores are the same
  // memory.  sh, maxB and maxQ describe the table the kernels see; user_* what the caller sees.
  int split;
  bool mfma;  // the shape runs on the matrix-core kernels (and they are not switched off)
  int64_t user_maxB, user_N;
  int user_D;
  Shape sh;
  int64_t maxB, maxQ;
  int sortBlocksMax, segBlocksMax, uBlocksMax, qBlocksMax, tilesMax;
  int64_t maxChunk3, maxChunk2;
  int keyBits, passes, bitsPerPass;
  // single-wavefront blocks of the per-chunk matrix-core kernels that the device holds at once
  // (forward, backward); asked of the runtime at the first launch, 0 until then
  mutable int unit_slots[2] = {0, 0};
};

// The by-i3 chunks are put in prefix order only when the prefix products of a batch of B ids can
// exceed one XCD's L2 (4 MiB); below that the gathers hit the L2 in any order.
inline bool chunks_ordered(const Plan& pl, int64_t B) {
  const int64_t q = B < pl.maxQ ? B : pl.maxQ;
  return q * pl.sh.PN * 4 > (int64_t)4 << 20;
}

enum KernelSlot {
  kSlotSortHist = 0,
  kSlotSortScan,
  kSlotSortScatter,
  kSlotSegCount,
  kSlotSegWrite,
  kSlotGroup,
  kSlotPrefixFwd,
  kSlotRowFwd,
  kSlotGsum,
  kSlotGsumFix,
  kSlotUBwd,
  kSlotDg3,
  kSlotPrefixBwd,
  kSlotSgd,
  kSlotEventPair,  // an event pair with nothing between: the cost the timing itself adds to a slot
  kSlotCount
};

}  // namespace ttemb

// Index pipeline of the TT-embedding forward pass (gfx950).
//
//   ids --split--> sort keys --stable LSD radix sort--> sorted slots
//       --segment scan--> unique ids (U) and unique (i1,i2) prefixes (Q) with their extents
//       --stable bucket passes--> unique ids grouped by i3, prefixes grouped by i2
//
// The split is i1 = i/(n2 n3), i2 = (i/n3) mod n2, i3 = i mod n3 (paper Section 4.2).  Sorting by
// the id itself makes every sharing level of the paper's Fig. "node-index" a contiguous run: equal
// ids, ids with a common (i1,i2) prefix (they share G1[i1] G2[i2]), ids with a common i1.
// Everything here is integer work and is bit-exact; all orders are stable, so the floating-point
// sums that later follow these lists are formed in a fixed order.
#include <algorithm>

#include "tt_emb_internal.h"

namespace ttemb {

__device__ __forceinline__ uint32_t key_of_id(const IdSource& src, int idx, uint32_t N) {
  int pos = idx, slab = 0;
  if (src.split > 1) {
    pos = idx / src.split;
    slab = idx - pos * src.split;
  }
  int64_t id = src.ids != nullptr ? src.ids[pos] : src.base + pos;
  if (src.reindex != nullptr) {
    // node re-indexing (paper Section 4.2: ids renumbered so that a partition's nodes are
    // consecutive): one gather in front of the split
    if ((uint64_t)id >= (uint64_t)src.n_ids) return N;
    id = src.reindex[id];
  }
  // ids outside the table (negative ones included) become the sentinel N and sort to the end
  if ((uint64_t)id >= (uint64_t)src.rows) return N;
  if (src.split > 1) {
    // first-core index i1 -> split*i1 + slab, the other two coordinates stay
    const int64_t i1 = id / src.n23;
    id += ((int64_t)(src.split - 1) * i1 + slab) * src.n23;
  }
  return (uint32_t)id;
}

// band of the prefix range [0, Q) that prefix q falls in (single precision: bands only order a
// schedule, and both users call this one function)
__device__ __forceinline__ int chunk_band(int q, int Q) {
  const float b = (float)max(q, 0) * ((float)kOrderBands / (float)max(Q, 1));
  return min((int)b, kOrderBands - 1);
}

// ---------------------------------------------------------------------------------------------
// block-wide helpers; ldsw holds at least one word per wavefront of the block

// Inclusive prefix sum over the wavefront: inside every row of 16 lanes with cross-lane moves in
// the vector ALU (row_shr by 1, 2, 4, 8; lanes without a source add zero), then the totals of the
// rows before a lane's own are added.
__device__ __forceinline__ uint32_t row_shr_or_zero(uint32_t v, int by) {
  // by is a compile-time constant after unrolling
  switch (by) {
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);
    case 4: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);
    default: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);
  }
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
  v += row_shr_or_zero(v, 1);
  v += row_shr_or_zero(v, 2);
  v += row_shr_or_zero(v, 4);
  v += row_shr_or_zero(v, 8);
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  const int row = lane / 16;
  return v + (row >= 1 ? r0 : 0u) + (row >= 2 ? r1 : 0u) + (row >= 3 ? r2 : 0u);
}

// Exclusive prefix of v over the block's threads; *total receives the block sum.
__device__ __forceinline__ uint32_t block_exclusive_scan_value(uint32_t v, uint32_t* ldsw,
                                                               uint32_t* total) {
  const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  const uint32_t incl = wave_inclusive_scan(v, lane);
  if (lane == kWave - 1) ldsw[w] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int k = 0; k < nw; ++k) {
    const uint32_t t = ldsw[k];
    base += (k < w) ? t : 0u;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return base + incl - v;
}

// In-place exclusive scan of an LDS array arr[0..n), n <= kMaxBins; returns the total.
__device__ uint32_t block_exclusive_scan(uint32_t* arr, int n, uint32_t* ldsw) {
  const int tid = threadIdx.x, nt = blockDim.x;
  const int per = (n + nt - 1) / nt;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  uint32_t s = 0;
  for (int i = lo; i < hi; ++i) s += arr[i];
  uint32_t total;
  uint32_t run = block_exclusive_scan_value(s, ldsw, &total);
  for (int i = lo; i < hi; ++i) {
    const uint32_t t = arr[i];
    arr[i] = run;
    run += t;
  }
  __syncthreads();
  return total;
}

// Lanes of a wavefront that hold the same digit (among lanes with valid set).  One ballot per bit of
// the widest digit (higher bits are zero everywhere and cost nothing but their ballot): a lane
// collects the lanes that differ from it in some bit as (vote xor own bit replicated).
constexpr int kMaxBits = 11;
static_assert((1 << kMaxBits) == kMaxBins, "digits have at most kMaxBits bits");
__device__ __forceinline__ unsigned long long match_digit(int digit, bool valid) {
  const int d = valid ? digit : 0;
  uint32_t lo = 0u, hi = 0u;
#pragma unroll
  for (int bit = 0; bit < kMaxBits; ++bit) {
    const int t = (d << (31 - bit)) >> 31;  // 0 or -1
    const unsigned long long vote = __ballot(t < 0);
    lo |= (uint32_t)vote ^ (uint32_t)t;
    hi |= (uint32_t)(vote >> 32) ^ (uint32_t)t;
  }
  return ~(((unsigned long long)hi << 32) | lo) & __ballot(valid);
}

struct alignas(16) ScatterLds {
  // per-wavefront bucket counts, later block-local output offsets; two 16-bit buckets per word
  // (a wavefront owns 256 items and a block 4096, so both fit)
  uint32_t wh[kSortWaves][kMaxBins / 2];
  uint32_t tot[kMaxBins];  // bucket totals, then this block's first output per bucket
  uint32_t aux[kMaxBins];  // chunks per bucket, then first chunk per bucket
  uint32_t base[kMaxBins]; // first output of every bucket (all blocks), for chunked passes
  uint32_t ldsw[kSortWaves];
};

constexpr int kSteps = kSortWaveItems / kWave;  // items per lane
static_assert((kChunk2 & (kChunk2 - 1)) == 0 && (kChunk3 & (kChunk3 - 1)) == 0 &&
                  (kChunk3Min & (kChunk3Min - 1)) == 0,
              "chunk sizes are powers of two: positions inside a bucket are cut with shifts");

// One block's share of a stable counting-sort pass over n_items items (block blk owns items
// [blk*kSortItems, +kSortItems), wavefront w of it the w-th sixteenth).  With tot != nullptr,
// cnt[b][bin] holds, per bucket, the items of blocks before b and tot[bin] the bucket totals (both
// from a column-scan kernel over the blocks' histograms); with tot == nullptr, cnt holds the
// blocks' own histograms and every block adds up its columns itself (cheaper than one more launch
// when there are few blocks).
// ItemOps: Item load(int idx); int digit(Item); void emit(uint32_t pos, Item); and, for chunked
// passes, void emit_chunked(uint32_t pos, uint32_t chunk, uint32_t t, Item): item is the t-th of
// chunk `chunk` (its record goes to chunk*chunk_size + t of a per-chunk table).
// With starts != nullptr the pass also publishes the bucket offsets (bins+1 entries, by block 0)
// and, for chunk > 0, cuts every bucket into chunks of at most `chunk` items: chunk_desc[c] =
// {bucket, first item, item count, 0} for all chunks c in bucket order, chunk_starts[bucket] the
// first chunk of each bucket (bins+1 entries), *n_chunks the number of chunks.
template <class ItemOps>
__device__ void stable_scatter_block(ScatterLds& L, int blk, int n_items, int bins,
                                     const uint32_t* __restrict__ cnt,
                                     const uint32_t* __restrict__ tot, ItemOps ops, int* starts,
                                     int chunk, int* chunk_starts, int4* chunk_desc,
                                     int* n_chunks) {
  const int tid = threadIdx.x;
  const int nblk = (n_items + kSortItems - 1) / kSortItems;
  const bool publishes = (starts != nullptr && blk == 0);
  const int chunk_sh = chunk > 0 ? 31 - __clz(chunk) : 0;  // chunk sizes are powers of two
  if (blk >= nblk && !publishes) return;  // uniform for the whole block

  // items first: their loads overlap the table work below
  const int w = tid / kWave, lane = tid % kWave;
  const int wbase = blk * kSortItems + w * kSortWaveItems;
  typename ItemOps::Item items[kSteps];
  int digits[kSteps];
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int idx = wbase + step * kWave + lane;
    items[step] = ops.load(idx < n_items ? idx : 0);
  }
  uint32_t before[kMaxBins / kSortThreads];  // items of my buckets in earlier blocks
#pragma unroll
  for (int k = 0; k < kMaxBins / kSortThreads; ++k) {
    const int bin = tid + k * kSortThreads;
    const int bc = min(bin, bins - 1);
    uint32_t total;
    if (tot != nullptr) {
      total = tot[bc];
      before[k] = cnt[(size_t)blk * bins + bc];
    } else {
      // column sums over the blocks' histograms, kFoldRows rows in flight
      uint32_t bsum = 0, tsum = 0;
      for (int b0 = 0; b0 < nblk; b0 += kFoldRows) {
        uint32_t v[kFoldRows];
#pragma unroll
        for (int j = 0; j < kFoldRows; ++j) v[j] = cnt[(size_t)min(b0 + j, nblk - 1) * bins + bc];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < kFoldRows; ++j) {
          const uint32_t x = (b0 + j < nblk) ? v[j] : 0u;
          tsum += x;
          bsum += (b0 + j < blk) ? x : 0u;
        }
      }
      total = tsum;
      before[k] = bsum;
    }
    if (bin < bins) {
      L.tot[bin] = total;
      if (chunk > 0) L.aux[bin] = (total + chunk - 1) >> chunk_sh;
    }
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the loads together: their latencies overlap
#pragma unroll
  for (int step = 0; step < kSteps; ++step) digits[step] = ops.digit(items[step]);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int step = 0; step < kSteps; ++step)
    if (wbase + step * kWave + lane >= n_items) digits[step] = -1;
  __syncthreads();
  const uint32_t total_items = block_exclusive_scan(L.tot, bins, L.ldsw);
  if (chunk > 0) {
    for (int bin = tid; bin < bins; bin += kSortThreads) L.base[bin] = L.tot[bin];
  }
  if (starts != nullptr) {
    if (publishes) {
      for (int bin = tid; bin < bins; bin += kSortThreads) starts[bin] = (int)L.tot[bin];
      if (tid == 0) starts[bins] = (int)total_items;
    }
    if (chunk > 0) {
      // every participating block takes a share of the chunk descriptors
      const uint32_t total_chunks = block_exclusive_scan(L.aux, bins, L.ldsw);
      if (publishes) {
        for (int bin = tid; bin < bins; bin += kSortThreads) chunk_starts[bin] = (int)L.aux[bin];
        if (tid == 0) {
          chunk_starts[bins] = (int)total_chunks;
          *n_chunks = (int)total_chunks;
        }
      }
      const int nshare = max(nblk, 1);
      for (uint32_t c = (uint32_t)blk * kSortThreads + tid; c < total_chunks;
           c += (uint32_t)nshare * kSortThreads) {
        int lo = 0, hi = bins;  // last bucket whose first chunk is <= c
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (L.aux[mid] <= c) lo = mid; else hi = mid;
        }
        const uint32_t first = L.tot[lo];
        const uint32_t end = (lo + 1 < bins) ? L.tot[lo + 1] : total_items;
        const uint32_t k0 = first + (c - L.aux[lo]) * (uint32_t)chunk;
        chunk_desc[c] = make_int4(lo, (int)k0, (int)min((uint32_t)chunk, end - k0), 0);
      }
    }
  }
  if (blk >= nblk) return;
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kMaxBins / kSortThreads; ++k) {
    const int bin = tid + k * kSortThreads;
    if (bin < bins) L.tot[bin] += before[k];
  }
  // every wavefront clears its own counters, 16 bytes per lane and write (no barrier: nobody else
  // touches them before the next one)
  const int words = (bins + 1) / 2;
  for (int i = lane; i < (words + 3) / 4; i += kWave) ((uint4*)L.wh[w])[i] = make_uint4(0u, 0u, 0u, 0u);

  // Each wavefront walks its items in order, 64 at a time.  Lanes holding the same digit find each
  // other by ballots; the lowest of them advances the wavefront's bucket counter for all, which
  // gives every item its rank among the wavefront's items of that bucket.
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  uint32_t rank[kSteps];
  unsigned long long peers[kSteps];
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const bool valid = digits[step] >= 0;
    peers[step] = 0ull;
    if (__ballot(valid) != 0ull) peers[step] = match_digit(digits[step], valid);  // wave-uniform
  }
  // the counter updates of the steps go out back to back (the LDS keeps a wavefront's atomics in
  // program order, which is what makes the ranks stable), their results are picked up afterwards
  uint32_t old[kSteps];
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int digit = digits[step];
    old[step] = 0;
    if (digit >= 0 && lane == __ffsll((long long)peers[step]) - 1)
      old[step] = atomicAdd(&L.wh[w][digit >> 1], (uint32_t)__popcll(peers[step]) << (16 * (digit & 1)));
  }
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int digit = digits[step];
    const int leader = digit >= 0 ? (__ffsll((long long)peers[step]) - 1) : lane;
    rank[step] = ((__shfl(old[step], leader) >> (16 * (digit & 1))) & 0xffffu) +
                 (uint32_t)__popcll(peers[step] & lt_mask);
  }
  __syncthreads();
  // per bucket: counts of the wavefronts -> offsets inside the block (one thread per word)
  for (int word = tid; word < words; word += kSortThreads) {
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int k = 0; k < kSortWaves; ++k) {
      const uint32_t c = L.wh[k][word];
      L.wh[k][word] = lo | (hi << 16);
      lo += c & 0xffffu;
      hi += c >> 16;
    }
  }
  __syncthreads();
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int digit = digits[step];
    if (digit >= 0) {
      const uint32_t off = (L.wh[w][digit >> 1] >> (16 * (digit & 1))) & 0xffffu;
      const uint32_t pos = L.tot[digit] + off + rank[step];
      if constexpr (ItemOps::kChunked) {
        const uint32_t in_bucket = pos - L.base[digit];
        ops.emit_chunked(pos, L.aux[digit] + (in_bucket >> chunk_sh), in_bucket & (uint32_t)(chunk - 1),
                         items[step]);
      } else {
        ops.emit(pos, items[step]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// LSD radix sort of (key = id or sentinel, value = batch position)

struct KV {
  uint32_t key, val;
};

template <bool FROM_IDS>
struct SortOps {
  using Item = KV;
  static constexpr bool kChunked = false;
  IdSource src;
  const uint32_t* kin;
  const uint32_t* vin;
  uint32_t* kout;
  uint32_t* vout;
  uint32_t N;
  int shift;
  uint32_t mask;
  __device__ Item load(int idx) const {
    if (FROM_IDS) return KV{key_of_id(src, idx, N), (uint32_t)idx};
    return KV{kin[idx], vin[idx]};
  }
  __device__ int digit(Item it) const { return (int)((it.key >> shift) & mask); }
  __device__ void emit(uint32_t pos, Item it) const {
    kout[pos] = it.key;
    vout[pos] = it.val;
  }
};

// Bucket counts of one radix digit per block of kSortItems items.  Equal digits inside a
// wavefront step are counted with one LDS atomic (a hot id would otherwise serialise thousands of
// them).  The first pass also clears the tables that later kernels of the same forward add into.
template <bool FROM_IDS>
__global__ __launch_bounds__(kSortThreads) void k_sort_hist(
    IdSource src, const uint32_t* __restrict__ kin, int B, uint32_t N, int shift,
    int bits, uint32_t* __restrict__ cnt, uint32_t* zero_a, int zero_a_n, uint32_t* zero_b,
    int zero_b_n, uint32_t* zero_c, int zero_c_n, Counters* ctr) {
  __shared__ uint32_t h[kMaxBins];
  const int tid = threadIdx.x, bins = 1 << bits;
  const uint32_t mask = (uint32_t)bins - 1u;
  const int w = tid / kWave, lane = tid % kWave;
  const int wbase = blockIdx.x * kSortItems + w * kSortWaveItems;
  uint32_t keys[kSteps];
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int idx = wbase + step * kWave + lane;
    const int ic = min(idx, B - 1);
    keys[step] = FROM_IDS ? key_of_id(src, ic, N) : kin[ic];
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the loads together: their latencies overlap
  if (FROM_IDS) {
    const int gtid = blockIdx.x * kSortThreads + tid, gn = gridDim.x * kSortThreads;
    for (int i = gtid; i < zero_a_n; i += gn) zero_a[i] = 0u;
    for (int i = gtid; i < zero_b_n; i += gn) zero_b[i] = 0u;
    for (int i = gtid; i < zero_c_n; i += gn) zero_c[i] = 0u;
    if (gtid == 0) {
      ctr->err = 0;
      ctr->n_split = 0;
    }
  }
  for (int i = tid; i < bins; i += kSortThreads) h[i] = 0u;
  __syncthreads();
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    const int idx = wbase + step * kWave + lane;
    const bool valid = idx < B;
    if (__ballot(valid) == 0ull) continue;
    const int digit = (int)((keys[step] >> shift) & mask);
    const unsigned long long peers = match_digit(digit, valid);
    if (valid && lane == __ffsll((long long)peers) - 1)
      atomicAdd(&h[digit], (uint32_t)__popcll(peers));
  }
  __syncthreads();
  for (int i = tid; i < bins; i += kSortThreads) cnt[(size_t)blockIdx.x * bins + i] = h[i];
}

template <bool FROM_IDS>
__global__ __launch_bounds__(kSortThreads) void k_sort_scatter(SortOps<FROM_IDS> ops, int B,
                                                               int bits,
                                                               const uint32_t* __restrict__ cnt,
                                                               const uint32_t* __restrict__ tot) {
  __shared__ ScatterLds L;
  stable_scatter_block(L, (int)blockIdx.x, B, 1 << bits, cnt, tot, ops, nullptr, 0, nullptr,
                       nullptr, nullptr);
}

// Turns the blocks' bucket counts cnt[b][bin] into counts of earlier blocks (exclusive scan down
// each column) and leaves the column totals in tot[bin].  One thread per bucket.
__device__ __forceinline__ void column_scan(uint32_t* __restrict__ cnt, uint32_t* __restrict__ tot,
                                            int nblk, int bins, int bin) {
  uint32_t run = 0;
  uint32_t* col = cnt + bin;
  int b2 = 0;
  for (; b2 + 16 <= nblk; b2 += 16) {
    uint32_t c[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) c[k] = col[(size_t)(b2 + k) * bins];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      col[(size_t)(b2 + k) * bins] = run;
      run += c[k];
    }
  }
  for (; b2 < nblk; ++b2) {
    const uint32_t c = col[(size_t)b2 * bins];
    col[(size_t)b2 * bins] = run;
    run += c;
  }
  tot[bin] = run;
}

constexpr int kScanThreads = 64;

__global__ __launch_bounds__(kScanThreads) void k_sort_colscan(uint32_t* __restrict__ cnt,
                                                               uint32_t* __restrict__ tot, int nblk,
                                                               int bins) {
  const int bin = blockIdx.x * kScanThreads + threadIdx.x;
  if (bin < bins) column_scan(cnt, tot, nblk, bins, bin);
}

// ---------------------------------------------------------------------------------------------
// Segment discovery over the sorted keys

struct SegFlags {
  uint32_t key[4], prev[4];
  bool valid[4], newu[4], newq[4], last_valid[4], single[4], split[4];
};

__device__ __forceinline__ SegFlags seg_flags(const uint32_t* __restrict__ skey, int B, uint32_t N,
                                              uint32_t n3, int s0) {
  SegFlags f;
  uint32_t k[6];  // keys of slots s0-1 .. s0+4
#pragma unroll
  for (int j = 0; j < 6; ++j) {
    const int s = s0 - 1 + j;
    k[j] = (s >= 0 && s < B) ? skey[s] : 0xffffffffu;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int s = s0 + j;
    const uint32_t key = k[j + 1], prev = k[j], next = k[j + 2];
    f.key[j] = key;
    f.prev[j] = prev;
    f.valid[j] = (s < B) && (key < N);
    const bool first = (s == 0);
    // a new entry: a new id, or the next kEntrySlots piece of a long run of one id
    const bool cut = (s % kEntrySlots) == 0;
    f.newu[j] = f.valid[j] && (first || key != prev || cut);
    f.split[j] = f.valid[j] && !first && key == prev && cut;
    f.newq[j] = f.valid[j] && (first || (key / n3) != (prev / n3));
    f.last_valid[j] = f.valid[j] && !(next < N);
    // the entry holds exactly one slot: its gradient row is read where it lies
    f.single[j] = f.newu[j] && (next != key || ((s + 1) % kEntrySlots) == 0);
  }
  return f;
}

__global__ __launch_bounds__(kSegThreads) void k_seg_count(const uint32_t* __restrict__ skey, int B,
                                                           uint32_t N, uint32_t n3,
                                                           uint32_t* __restrict__ seg_nu,
                                                           uint32_t* __restrict__ seg_nq) {
  __shared__ uint32_t lds4[kSegThreads / kWave];
  const SegFlags f = seg_flags(skey, B, N, n3, (int)blockIdx.x * kSegItems + (int)threadIdx.x * 4);
  uint32_t cu = 0, cq = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    cu += f.newu[j];
    cq += f.newq[j];
  }
  uint32_t tu, tq;
  block_exclusive_scan_value(cu, lds4, &tu);
  block_exclusive_scan_value(cq, lds4, &tq);
  if (threadIdx.x == 0) {
    seg_nu[blockIdx.x] = tu;
    seg_nq[blockIdx.x] = tq;
  }
}

// Numbers the unique ids and prefixes in sorted order, records their extents and coordinates, and
// counts them per (block of 4096, i3) resp. (block of 4096, i2) for the grouping pass and per i1.
// u_code[u] says where the gradient row of unique id u will be found: >= 0 is the batch position
// of its only occurrence, -(u+1) means "row u of the per-id sums".
__global__ __launch_bounds__(kSegThreads) void k_seg_write(
    const uint32_t* __restrict__ skey, const uint32_t* __restrict__ perm, int B, Shape sh,
    const uint32_t* __restrict__ seg_nu, const uint32_t* __restrict__ seg_nq, int* __restrict__ s_u,
    int4* __restrict__ s_rec, int* __restrict__ u_rs, int* __restrict__ u_i3, int* __restrict__ u_q, int* __restrict__ u_code,
    int* __restrict__ q_us, int* __restrict__ q_i1, int* __restrict__ q_i2,
    uint32_t* __restrict__ cnt3, uint32_t* __restrict__ cnt2, int* __restrict__ g1_first,
    int* __restrict__ g1_end, Counters* __restrict__ ctr) {
  __shared__ uint32_t lds4[kSegThreads / kWave];
  const int tid = threadIdx.x, blk = blockIdx.x;
  const int s0 = blk * kSegItems + tid * 4;
  const SegFlags f = seg_flags(skey, B, sh.N, sh.n3, s0);
  uint32_t bpos[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) bpos[j] = (s0 + j < B) ? perm[s0 + j] : 0u;
  uint32_t pu = 0, pq = 0;
  for (int b2 = tid; b2 < blk; b2 += kSegThreads) {
    pu += seg_nu[b2];
    pq += seg_nq[b2];
  }
  uint32_t offu, offq, dummy;
  block_exclusive_scan_value(pu, lds4, &offu);
  block_exclusive_scan_value(pq, lds4, &offq);

  uint32_t cu = 0, cq = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    cu += f.newu[j];
    cq += f.newq[j];
  }
  uint32_t ru = offu + block_exclusive_scan_value(cu, lds4, &dummy);  // unique ids before my slots
  uint32_t rq = offq + block_exclusive_scan_value(cq, lds4, &dummy);

  if (blk == 0 && tid == 0 && !f.valid[0]) {  // no in-range id at all
    ctr->U = 0;
    ctr->Q = 0;
    ctr->nvalid = 0;
    u_rs[0] = 0;
    q_us[0] = 0;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int s = s0 + j;
    if (s >= B) break;
    if (!f.valid[j]) {
      s_u[s] = -1;
      s_rec[s] = make_int4(-1, (int)bpos[j], 0, 0);
      continue;
    }
    ru += f.newu[j];
    rq += f.newq[j];
    const int u = (int)ru - 1, q = (int)rq - 1;
    s_u[s] = u;
    const uint32_t k = f.key[j];
    // everything the row kernel needs about a slot in one record (one load instead of a chain)
    s_rec[s] = make_int4(u, (int)bpos[j], q, (int)(k % sh.n3));
    if (f.split[j]) atomicAdd(&ctr->n_split, 1);
    if (f.newu[j]) {
      const uint32_t i3 = k % sh.n3;
      u_rs[u] = s;
      u_i3[u] = (int)i3;
      u_q[u] = q;
      u_code[u] = f.single[j] ? (int)bpos[j] : -(u + 1);
      atomicAdd(&cnt3[(size_t)(u / kSortItems) * sh.n3 + i3], 1u);
    }
    if (f.newq[j]) {
      const uint32_t p = k / sh.n3;  // prefix number i1*n2 + i2
      const uint32_t i1 = p / sh.n2, i2 = p % sh.n2;
      q_us[q] = u;
      q_i1[q] = (int)i1;
      q_i2[q] = (int)i2;
      atomicAdd(&cnt2[(size_t)(q / kSortItems) * sh.n2 + i2], 1u);
      // prefixes are numbered in (i1,i2) order: an i1 owns prefixes [g1_first, g1_end)
      const uint32_t i1_before = (s == 0) ? 0xffffffffu : f.prev[j] / sh.n3 / sh.n2;
      if (i1_before != i1) {
        g1_first[i1] = q;
        if (s != 0) g1_end[i1_before] = q;
      }
    }
    if (f.last_valid[j]) {
      ctr->U = u + 1;
      ctr->Q = q + 1;
      ctr->nvalid = s + 1;
      u_rs[u + 1] = s + 1;
      q_us[q + 1] = u + 1;
      g1_end[k / sh.n3 / sh.n2] = q + 1;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Grouping: unique ids by i3 (for the G3 gradient), prefixes by i2 (for G2 and the prefix product)

// Unique ids by i3.  Besides the list, every chunk gets a table of its ids' records
// {gradient-row code, prefix}, so that the gradient kernels need no further look-ups.
struct GroupOps3 {
  struct Item {
    int u, i3, code, q;
  };
  static constexpr bool kChunked = true;
  const int* u_i3;
  const int* u_code;
  const int* u_q;
  int* list;
  int2* item;
  uint32_t* band_cnt;
  int Q;
  __device__ Item load(int idx) const { return Item{idx, u_i3[idx], u_code[idx], u_q[idx]}; }
  __device__ int digit(Item it) const { return it.i3; }
  __device__ void emit_chunked(uint32_t pos, uint32_t chunk, uint32_t t, Item it) const {
    list[pos] = it.u;
    item[(size_t)chunk * kChunk3 + t] = make_int2(it.code, it.q);
    // a chunk counts where it starts (only when a schedule will be built from the counts)
    if (band_cnt != nullptr && t == 0) atomicAdd(&band_cnt[chunk_band(it.q, Q)], 1u);
  }
};

// Prefixes by i2; chunk records are {prefix, i1, first unique id, one past its last unique id}.
struct GroupOps2 {
  struct Item {
    int q, i2, i1, u0, u1;
  };
  static constexpr bool kChunked = true;
  const int* q_i2;
  const int* q_i1;
  const int* q_us;
  int* list;
  int4* item;
  __device__ Item load(int idx) const {
    return Item{idx, q_i2[idx], q_i1[idx], q_us[idx], q_us[idx + 1]};
  }
  __device__ int digit(Item it) const { return it.i2; }
  __device__ void emit_chunked(uint32_t pos, uint32_t chunk, uint32_t t, Item it) const {
    list[pos] = it.q;
    item[(size_t)chunk * kChunk2 + t] = make_int4(it.q, it.i1, it.u0, it.u1);
  }
};

__global__ __launch_bounds__(kSortThreads) void k_group(
    Shape sh, int u_blocks, int chunk3, const uint32_t* __restrict__ cnt3,
    const uint32_t* __restrict__ cnt2, const int* __restrict__ u_i3, const int* __restrict__ u_code,
    const int* __restrict__ u_q, const int* __restrict__ q_i2, const int* __restrict__ q_i1,
    const int* __restrict__ q_us, int* g3_list, int* g3_start, int* c3_start, int4* c3_desc,
    int2* c3_item, int* g2_list, int* g2_start, int* c2_start, int4* c2_desc, int4* c2_item,
    uint32_t* band_cnt, Counters* ctr) {
  __shared__ ScatterLds L;
  if ((int)blockIdx.x < u_blocks) {
    GroupOps3 ops{u_i3, u_code, u_q, g3_list, c3_item, band_cnt, ctr->Q};
    stable_scatter_block(L, (int)blockIdx.x, ctr->U, (int)sh.n3, cnt3, nullptr, ops, g3_start,
                         chunk3, c3_start, c3_desc, &ctr->nchunk3);
  } else {
    GroupOps2 ops{q_i2, q_i1, q_us, g2_list, c2_item};
    stable_scatter_block(L, (int)blockIdx.x - u_blocks, ctr->Q, (int)sh.n2, cnt2, nullptr, ops,
                         g2_start, kChunk2, c2_start, c2_desc, &ctr->nchunk2);
  }
}

// The by-i3 chunks in the order of the prefix of their first id, bucketed into kOrderBands bands of
// the prefix range (the order inside a band is whatever the atomics give).  The G3-gradient step
// gathers one prefix product per id: walking the chunks in this order makes neighbouring
// wavefronts gather neighbouring products.  Only the schedule depends on it, never a result.
// The grouping kernel has counted the chunks per band; every block scans those counts for itself.
__global__ __launch_bounds__(kSortThreads) void k_chunk_order(const int2* __restrict__ c3_item,
                                                             const uint32_t* __restrict__ band_cnt,
                                                             uint32_t* __restrict__ band_cur,
                                                             int* __restrict__ c3_order,
                                                             const Counters* __restrict__ ctr) {
  __shared__ uint32_t band_at[kOrderBands];
  __shared__ uint32_t ldsw[kSortWaves];
  static_assert(kOrderBands == kSortThreads, "one band per thread");
  const int tid = threadIdx.x, n = ctr->nchunk3, c = blockIdx.x * kSortThreads + tid;
  if ((int)blockIdx.x * kSortThreads >= n) return;
  const int q = c < n ? c3_item[(size_t)c * kChunk3].y : 0;
  band_at[tid] = band_cnt[tid];
  __syncthreads();
  block_exclusive_scan(band_at, kOrderBands, ldsw);
  if (c < n) {
    const int b = chunk_band(q, ctr->Q);
    c3_order[band_at[b] + atomicAdd(&band_cur[b], 1u)] = c;
  }
}

// ---------------------------------------------------------------------------------------------
// host-side launchers

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

void launch_sort_pass(const Plan& pl, const Workspace& ws, const IdSource& src, int B, int pass,
                      hipStream_t st, int which /*0 = histogram, 1 = scatter, 2 = column scan*/) {
  const int blocks = cdiv(B, kSortItems);
  const int shift = pass * pl.bitsPerPass;
  const int bits = std::min(pl.bitsPerPass, pl.keyBits - shift);
  const uint32_t N = pl.sh.N;
  // with few blocks every scatter block adds up the histogram columns itself: no scan launch
  const bool folded = blocks <= kFoldScanBlocks;
  const uint32_t* tot = folded ? nullptr : ws.tot;
  if (which == 2) {
    if (!folded)
      k_sort_colscan<<<cdiv(1 << bits, kScanThreads), kScanThreads, 0, st>>>(ws.cnt, ws.tot, blocks,
                                                                           1 << bits);
    return;
  }
  if (pass == 0) {
    if (which == 0) {
      k_sort_hist<true><<<blocks, kSortThreads, 0, st>>>(
          src, nullptr, B, N, shift, bits, ws.cnt, ws.cnt3, pl.uBlocksMax * (int)pl.sh.n3, ws.cnt2,
          pl.qBlocksMax * (int)pl.sh.n2, (uint32_t*)ws.g1_first,
          2 * (int)pl.sh.n1 + 2 * kOrderBands, ws.ctr);
    } else {
      SortOps<true> ops{src, nullptr, nullptr, ws.key[0], ws.val[0], N, shift, (1u << bits) - 1u};
      k_sort_scatter<true><<<blocks, kSortThreads, 0, st>>>(ops, B, bits, ws.cnt, tot);
    }
  } else {
    const int from = (pass - 1) & 1, dst = pass & 1;
    if (which == 0) {
      k_sort_hist<false><<<blocks, kSortThreads, 0, st>>>(IdSource{}, ws.key[from], B, N, shift, bits,
                                                          ws.cnt, nullptr, 0, nullptr, 0, nullptr, 0,
                                                          ws.ctr);
    } else {
      SortOps<false> ops{IdSource{}, ws.key[from], ws.val[from], ws.key[dst], ws.val[dst], N, shift,
                         (1u << bits) - 1u};
      k_sort_scatter<false><<<blocks, kSortThreads, 0, st>>>(ops, B, bits, ws.cnt, tot);
    }
  }
}

void launch_seg_count(const Plan& pl, const Workspace& ws, int B, hipStream_t st) {
  const uint32_t* skey = ws.key[(pl.passes - 1) & 1];
  k_seg_count<<<cdiv(B, kSegItems), kSegThreads, 0, st>>>(skey, B, pl.sh.N, pl.sh.n3, ws.seg_nu,
                                                         ws.seg_nq);
}

void launch_seg_write(const Plan& pl, const Workspace& ws, int B, hipStream_t st) {
  const int f = (pl.passes - 1) & 1;
  k_seg_write<<<cdiv(B, kSegItems), kSegThreads, 0, st>>>(
      ws.key[f], ws.val[f], B, pl.sh, ws.seg_nu, ws.seg_nq, ws.s_u, ws.s_rec, ws.u_rs, ws.u_i3, ws.u_q,
      ws.u_code, ws.q_us, ws.q_i1, ws.q_i2, ws.cnt3, ws.cnt2, ws.g1_first, ws.g1_end, ws.ctr);
}

// which: 0 = both groupings and the chunk schedule; 1 = both groupings, no schedule (c3_order is
// not written: the gradient kernel then walks the by-i3 chunks in index order); 2 = prefixes by i2
// only (all a lookup needs)
void launch_group(const Plan& pl, const Workspace& ws, int B, hipStream_t st, int which) {
  // blocks are sized from upper bounds (U <= B, Q <= min(B, n1*n2)); surplus blocks return at once
  const int ub = which == 2 ? 0 : cdiv(B, kSortItems);
  const int qb = cdiv(std::min((int64_t)B, pl.maxQ), kSortItems);
  const bool ordered = which == 0 && chunks_ordered(pl, B);
  k_group<<<ub + qb, kSortThreads, 0, st>>>(pl.sh, ub, chunk3_fill(B), ws.cnt3, ws.cnt2, ws.u_i3, ws.u_code, ws.u_q, ws.q_i2, ws.q_i1,
                                           ws.q_us, ws.g3_list, ws.g3_start, ws.c3_start, ws.c3_desc,
                                           ws.c3_item, ws.g2_list, ws.g2_start, ws.c2_start,
                                           ws.c2_desc, ws.c2_item, ordered ? ws.band_cnt : nullptr, ws.ctr);
  if (ordered)
    k_chunk_order<<<cdiv(cdiv(B, chunk3_fill(B)) + (int64_t)pl.sh.n3, kSortThreads), kSortThreads, 0,
                    st>>>(
      ws.c3_item, ws.band_cnt, ws.band_cur, ws.c3_order, ws.ctr);
}

}  // namespace ttemb


// Matrix-core (MFMA, fp32) kernels for the table shapes d1 = d2 = 4, r1 = r2 = R in {16, 32, 64},
// d3 in {4, 8}: the partial product of a row is then 16 x R, and once ids that share an (i1,i2)
// prefix, an i2 or an i3 are stacked (paper Section 4.2: they share core slices) every step of the
// path is a dense contraction with a 16- or 32-wide side.
//
// Lane layouts used below (wave64):
//   v_mfma_f32_32x32x2f32   A[i][k]: i = lane%32, k = lane/32     B[k][j]: k = lane/32, j = lane%32
//                           D[i][j]: i = 8*(v/4) + 4*(lane/32) + v%4, j = lane%32, v = 0..15
//   v_mfma_f32_16x16x4f32   A[i][k]: i = lane%16, k = lane/16     B[k][j]: k = lane/16, j = lane%16
//                           D[i][j]: i = 4*(lane/16) + v, j = lane%16, v = 0..3
// The summation index k may be enumerated in any order as long as A and B agree, so each lane
// takes a contiguous run of k (vector loads) instead of the strided one the raw layout suggests.
#include <algorithm>
#include <type_traits>

#include "tt_emb_internal.h"

namespace ttemb {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kMThreads = 256;
constexpr int kMWaves = kMThreads / kWave;
// sorted slots per wavefront in the row kernel (lanes past it idle in the index steps): half a
// wavefront's worth keeps twice as many wavefronts in flight, which hides the store latency better
// sorted slots per wavefront in the row kernel: 16 for batches up to kRowSmallBatch rows (more
// wavefronts in flight: -2.6 us per step at 200,000 rows), 32 above (fewer repeated operand loads:
// -7 us at 500,000 rows)
constexpr int kRowSmallBatch = kSmallBatch;

__device__ __forceinline__ f16v mfma32(float a, float b, f16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ const float* grad_row_ptr(int code, const float* __restrict__ grad,
                                                     const float* __restrict__ gsum, int D) {
  // code >= 0: batch position of the id's only occurrence; else row -(code+1) of the per-id sums
  return code >= 0 ? grad + (size_t)code * D : gsum + (size_t)(-code - 1) * D;
}

typedef float f2 __attribute__((ext_vector_type(2)));

// Value of v in lane `src`, where src is the same for the whole wavefront (a scalar read, no LDS).
__device__ __forceinline__ int lane_value(int v, int src) {
  return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(src));
}

// One lane's share (VPL consecutive floats, VPL = 1 or 2) of a row, moved with a single
// non-temporal access: rows of out and grad_out are streamed once and should not displace the
// intermediates that the path does re-read.
template <int VPL>
__device__ __forceinline__ void stream_store(float* dst, const float* v) {
  if constexpr (VPL == 2) __builtin_nontemporal_store(f2{v[0], v[1]}, (f2*)dst);
  else __builtin_nontemporal_store(v[0], dst);
}
template <int VPL>
__device__ __forceinline__ void stream_load(const float* src, float* v) {
  if constexpr (VPL == 2) {
    const f2 t = __builtin_nontemporal_load((const f2*)src);
    v[0] = t.x;
    v[1] = t.y;
  } else {
    v[0] = __builtin_nontemporal_load(src);
  }
}

#define TT_ZERO16 {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}

// All kernels below are written as "issue every load of a work item, then compute": the loads of a
// phase sit in one straight-line block that ends in sched_barrier(0), so the compiler cannot sink
// them next to their uses (which would serialise their latencies); out-of-range lanes read a
// clamped, valid address and their values are discarded by a select.
#define TT_LOADS_DONE() __builtin_amdgcn_sched_barrier(0)

// ---------------------------------------------------------------------------------------------
// P_q = G1[i1] G2[i2] for the <= 16 prefixes of one by-i2 chunk: rows of up to eight G1 slices
// stacked (32 x R) times the chunk's G2 slice (R x 4R).  A work unit is (chunk, a share of the 4R
// output columns); one single-wavefront block per unit, so that the units spread evenly over all
// SIMDs.
// Units per chunk: two or four side by side over the 32-column tiles of the product (four shorten
// the kernel at rank 32 by a fifth; splitting the sixteen prefixes of a chunk over units as well
// only re-reads the G2 slice, which costs more than it gains).
// (At rank 128 a unit is a single 32 x 32 tile: its two operand strips alone are 128 registers.)
constexpr int pf_units(int R) { return R >= 128 ? 32 : R >= 32 ? 4 : 2; }

template <int R>
__global__ __launch_bounds__(kWave) void k_prefix_fwd_mfma(
    const float* __restrict__ g1, const float* __restrict__ g2, const int4* __restrict__ c2_item,
    const int4* __restrict__ c2_desc, float* __restrict__ P, float* __restrict__ Pt,
    int max_units, const Counters* __restrict__ ctr) {
  constexpr int W = 4 * R, PN = 16 * R, S1 = 4 * R, S2 = R * W, KH = R / 2, NT = W / 32;
  constexpr int kPfUnits = pf_units(R);
  constexpr int UC = kPfUnits < NT ? kPfUnits : NT;  // units side by side over the columns
  constexpr int UM = kPfUnits / UC;                  // 1: both row tiles in one unit, 2: one each
  constexpr int NTH = NT / UC, MTH = 2 / UM;         // column and row tiles of one unit
  const int lane = threadIdx.x, half = lane / 32, l32 = lane % 32;
  // The grid is sized from an upper bound of the chunk count (the real one is only known on the
  // device) and capped: a batch with far fewer chunks than its size allows would otherwise spend
  // its time dispatching empty blocks.  Blocks walk the units with the grid's stride.
  const int nchunk = ctr->nchunk2;
  auto do_unit = [&](const int unit) -> bool {  // false: no unit from here on has work
  const int c = unit / kPfUnits, sub = unit % kPfUnits;
  const int nt0 = (sub / UM) * NTH, mt0 = (sub % UM) * MTH;
  // the chunk's records and descriptor are read together with the count (max_units keeps the
  // reads inside the tables)
  const int4 item = c2_item[(size_t)c * kChunk2 + lane % kChunk2];
  const int4 desc = c2_desc[c];
  if (c >= nchunk) return false;
  const int bin = desc.x, cnt = desc.z;
  if (mt0 * 8 >= cnt) return true;  // the chunk has no prefix in this unit's row tile
  const float* Bm = g2 + (size_t)bin * S2 + (size_t)(KH * half) * W + nt0 * 32 + l32;
  float b[NTH][KH];
#pragma unroll
  for (int t = 0; t < NTH; ++t)
#pragma unroll
    for (int j = 0; j < KH; ++j) b[t][j] = Bm[(size_t)j * W + t * 32];
  const bool mine = lane < cnt;  // records past the chunk's count are unwritten
  const int myq = mine ? item.x : -1;
  const int myi1 = mine ? item.y : 0;
  float a[MTH][KH];
#pragma unroll
  for (int mt = 0; mt < MTH; ++mt) {
    const int ql = (mt0 + mt) * 8 + l32 / 4, j1 = l32 % 4;
    const int q = __shfl(myq, ql), i1 = __shfl(myi1, ql);
    const f4* src = (const f4*)(g1 + (size_t)i1 * S1 + j1 * R + KH * half);
#pragma unroll
    for (int j = 0; j < KH / 4; ++j) {
      f4 v = src[j];
      a[mt][4 * j + 0] = q >= 0 ? v.x : 0.f;
      a[mt][4 * j + 1] = q >= 0 ? v.y : 0.f;
      a[mt][4 * j + 2] = q >= 0 ? v.z : 0.f;
      a[mt][4 * j + 3] = q >= 0 ? v.w : 0.f;
    }
  }
  int qrow[MTH][4];  // prefix of accumulator rows v/4 of each row tile
#pragma unroll
  for (int mt = 0; mt < MTH; ++mt)
#pragma unroll
    for (int x = 0; x < 4; ++x) qrow[mt][x] = __shfl(myq, (mt0 + mt) * 8 + 2 * x + half);
  TT_LOADS_DONE();
#pragma unroll
  for (int t = 0; t < NTH; ++t) {
#pragma unroll
    for (int mt = 0; mt < MTH; ++mt) {
      if ((mt0 + mt) * 8 >= cnt) break;
      f16v acc = TT_ZERO16;
#pragma unroll
      for (int j = 0; j < KH; ++j) acc = mfma32(a[mt][j], b[t][j], acc);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int q = qrow[mt][v / 4];
        if (q >= 0) P[(size_t)q * PN + (v % 4) * W + (nt0 + t) * 32 + l32] = acc[v];
      }
      // Second copy for the G3-gradient step, which contracts over the 16 rows (j1,j2) of the
      // product: Pt[q][j2][b][j1], so that a lane of that step finds the four j1 of its (j2, b) in
      // one 16-byte word.  Accumulator elements 4x .. 4x+3 are j1 = 0..3 of one prefix at column
      // j2*R + b = (nt0+t)*32 + l32: one vector store per prefix, 512 contiguous bytes per half.
      if (Pt != nullptr) {
        const int col = (nt0 + t) * 32 + l32, j2 = col / R, b2 = col % R;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const int q = qrow[mt][x];
          if (q >= 0)
            *(f4*)&Pt[(size_t)q * PN + j2 * (4 * R) + b2 * 4] =
                f4{acc[4 * x], acc[4 * x + 1], acc[4 * x + 2], acc[4 * x + 3]};
        }
      }
    }
  }
  return true;
  };
  // rank 64 walks the units with the grid's stride (its grid is capped at what the device holds at
  // once); the other ranks have one block per possible unit
  if constexpr (R == 64) {
    for (int unit = blockIdx.x; unit < max_units; unit += gridDim.x)
      if (!do_unit(unit)) break;
  } else {
    if ((int)blockIdx.x < max_units) (void)do_unit((int)blockIdx.x);
  }
}

// ---------------------------------------------------------------------------------------------
// Gradients at prefix level for one by-i2 chunk (<= 16 prefixes q, Bm = G2[i2]).  Work units of a
// chunk, one single-wavefront block (or one turn of a block's loop) each:
//   row units  dg1part[q] = dPsum_q Bm^T for the first / second eight prefixes: their dPsum rows
//              stacked (32 x 4R) times Bm^T (4R x R); at rank 64 one unit per 32 of the R columns
//   col units  a share of the columns of part2[c] = sum_q G1[i1(q)]^T dPsum_q
//              ((R x 4 cnt) times (4 cnt x 4R)): halves; eighths at rank 64; at rank 128 halves of
//              the columns times halves of the rows
// (Rank 64 is cut finer because its batches often have few chunks: the launch then lasts as long
// as its longest unit, a chain of dependent load and multiply stages.)
constexpr int pb_col_units(int R) { return R == 64 ? 8 : 2; }  // units side by side over part2's columns
constexpr int pb_row_units(int R) { return R == 64 ? 4 : 2; }  // dg1part: two row tiles, at rank 64 times two column tiles
constexpr int pb_units(int R) { return pb_row_units(R) + pb_col_units(R) * (R >= 128 ? 2 : 1); }

template <int R>
__global__ __launch_bounds__(kWave) void k_prefix_bwd_mfma(
    const float* __restrict__ g1, const float* __restrict__ g2, const float* __restrict__ dPsum,
    const int4* __restrict__ c2_item, const int4* __restrict__ c2_desc, float* __restrict__ dg1part,
    float* __restrict__ part2, int max_units, Counters* __restrict__ ctr) {
  constexpr int W = 4 * R, PN = 16 * R, S1 = 4 * R, S2 = R * W;
  const int lane = threadIdx.x, half = lane / 32, l32 = lane % 32;
  constexpr int kPbUnits = pb_units(R);
  // capped grid, units walked with its stride (see k_prefix_fwd_mfma)
  const int nchunk = ctr->nchunk2;
  auto do_unit = [&](const int unit) -> bool {  // false: no unit from here on has work
  const int c = unit / kPbUnits, part = unit % kPbUnits;
  const int4 item = c2_item[(size_t)c * kChunk2 + lane % kChunk2];
  const int4 desc = c2_desc[c];
  if (c >= nchunk) return false;
  const int bin = desc.x, cnt = desc.z;
  constexpr int kRowUnits = pb_row_units(R);
  if (part < kRowUnits && (part % 2) == 1 && cnt <= 8) return true;
  const bool mine = lane < cnt;  // records past the chunk's count are unwritten
  const int myq = mine ? item.x : -1;
  const int myi1 = mine ? item.y : 0;
  const float* Bm = g2 + (size_t)bin * S2;

  if (part < kRowUnits) {
    constexpr int KB = W / 64;
    const int mt = part % 2;
    const int q = __shfl(myq, mt * 8 + l32 / 4), j1 = l32 % 4;
    const f4* arow = (const f4*)(dPsum + (size_t)(q >= 0 ? q : 0) * PN + j1 * W + 32 * half);
    int qrow[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) qrow[x] = __shfl(myq, mt * 8 + 2 * x + half);
    constexpr int NTU = (R + 31) / 32 / (kRowUnits / 2);  // 32-column tiles of this unit
#pragma unroll
    for (int nti = 0; nti < NTU; ++nti) {
      const int n = ((part / 2) * NTU + nti) * 32 + l32;
      const f4* brow = (const f4*)(Bm + (size_t)(n < R ? n : 0) * W + 32 * half);
      f4 av[2][8], bv[2][8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        av[0][j] = arow[j];
        bv[0][j] = brow[j];
      }
      TT_LOADS_DONE();
      f16v acc = TT_ZERO16;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        if (kb + 1 < KB) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            av[(kb + 1) & 1][j] = arow[(kb + 1) * 16 + j];
            bv[(kb + 1) & 1][j] = brow[(kb + 1) * 16 + j];
          }
          TT_LOADS_DONE();
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          f4 x = av[kb & 1][j], y = bv[kb & 1][j];
          if (q < 0) x = f4{0.f, 0.f, 0.f, 0.f};
          if (n >= R) y = f4{0.f, 0.f, 0.f, 0.f};
          acc = mfma32(x.x, y.x, acc);
          acc = mfma32(x.y, y.y, acc);
          acc = mfma32(x.z, y.z, acc);
          acc = mfma32(x.w, y.w, acc);
        }
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int qv = qrow[v / 4];
        if (qv >= 0 && n < R) dg1part[(size_t)qv * S1 + (v % 4) * R + n] = acc[v];
      }
    }
  } else {
    constexpr int MSPLIT = R >= 128 ? 2 : 1;                // units over the rows of part2
    constexpr int CU = pb_col_units(R);
    constexpr int MT = (R + 31) / 32 / MSPLIT, NT = W / 32, NTH = NT / CU;
    static_assert(NT % CU == 0, "column tiles divide evenly over the units");
    const int nt0 = ((part - kRowUnits) % CU) * NTH;
    const int mrow0 = ((part - kRowUnits) / CU) * MT * 32;  // first row of this unit
    int qh[8], ih[8];  // the eight prefixes whose rows this half of the wavefront feeds as k
#pragma unroll
    for (int jq = 0; jq < 8; ++jq) {
      qh[jq] = __shfl(myq, 8 * half + jq);
      ih[jq] = __shfl(myi1, 8 * half + jq);
    }
    float a[MT][32];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mrow0 + mt * 32 + l32;
#pragma unroll
      for (int j = 0; j < 32; ++j) a[mt][j] = g1[(size_t)ih[j / 4] * S1 + (j % 4) * R + (m < R ? m : 0)];
    }
    float b[2][32];
#pragma unroll
    for (int j = 0; j < 32; ++j)
      b[0][j] = dPsum[(size_t)(qh[j / 4] >= 0 ? qh[j / 4] : 0) * PN + (j % 4) * W + nt0 * 32 + l32];
    TT_LOADS_DONE();
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mrow0 + mt * 32 + l32;
#pragma unroll
      for (int j = 0; j < 32; ++j) a[mt][j] = (qh[j / 4] >= 0 && m < R) ? a[mt][j] : 0.f;
    }
#pragma unroll
    for (int t = 0; t < NTH; ++t) {
      const int n = (nt0 + t) * 32 + l32;
      if (t + 1 < NTH) {
#pragma unroll
        for (int j = 0; j < 32; ++j)
          b[(t + 1) & 1][j] =
              dPsum[(size_t)(qh[j / 4] >= 0 ? qh[j / 4] : 0) * PN + (j % 4) * W + n + 32];
        TT_LOADS_DONE();
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        f16v acc = TT_ZERO16;
#pragma unroll
        for (int j = 0; j < 32; ++j) acc = mfma32(a[mt][j], b[t & 1][j], acc);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int mrow = mrow0 + mt * 32 + 8 * (v / 4) + 4 * half + (v % 4);
          if (mrow < R) part2[(size_t)c * S2 + (size_t)mrow * W + n] = acc[v];
        }
      }
    }
  }
  return true;
  };
  // rank 64 walks the units with the grid's stride (its grid is capped at what the device holds at
  // once); the other ranks have one block per possible unit
  if constexpr (R == 64) {
    for (int unit = blockIdx.x; unit < max_units; unit += gridDim.x)
      if (!do_unit(unit)) break;
  } else {
    if ((int)blockIdx.x < max_units) (void)do_unit((int)blockIdx.x);
  }
}

// ---------------------------------------------------------------------------------------------
// dPsum_q = sum over the unique ids u of prefix q of g_u G3[i3(u)]^T  (16 x D3 times D3 x R).
// One wavefront per prefix; the ids of a prefix extend the contraction index, UB at a time.
template <int R, int D3>
__device__ __forceinline__ void u_bwd_role(
    int block, int nblocks, const float* __restrict__ g3, const float* __restrict__ grad,
    const float* __restrict__ gsum, const int* __restrict__ u_code, const int* __restrict__ u_i3,
    const int* __restrict__ q_us, float* __restrict__ dPsum, const Counters* __restrict__ ctr) {
  constexpr int PN = 16 * R, S3 = R * D3, D = 16 * D3, NT = R / 16, KS = D3 / 4, UB = 4;
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int l16 = lane % 16, kg = lane / 16;
  const int Q = ctr->Q;
  for (int q = block * kMWaves + w; q < Q; q += nblocks * kMWaves) {
    const int u0 = q_us[q], u1 = q_us[q + 1];
    f4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
    for (int ub = u0; ub < u1; ub += kWave) {
      const int n = min(kWave, u1 - ub);
      const int myi3 = u_i3[ub + min(lane, n - 1)];
      const int mycode = u_code[ub + min(lane, n - 1)];
      // UBX ids per round: their operand loads are in flight together
      auto round = [&](auto ubx, int i0) {
        constexpr int UBX = decltype(ubx)::value;
        float a[UBX][KS], b[UBX][NT][KS];
#pragma unroll
        for (int x = 0; x < UBX; ++x) {
          const int i = min(i0 + x, n - 1);
          const float* gp = grad_row_ptr(lane_value(mycode, i), grad, gsum, D) + l16 * D3 + KS * kg;
          const float* cp = g3 + (size_t)lane_value(myi3, i) * S3 + l16 * D3 + KS * kg;
#pragma unroll
          for (int s = 0; s < KS; ++s) a[x][s] = gp[s];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int s = 0; s < KS; ++s) b[x][nt][s] = cp[nt * 16 * D3 + s];
        }
        TT_LOADS_DONE();
#pragma unroll
        for (int x = 0; x < UBX; ++x) {
          const bool on = i0 + x < n;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int s = 0; s < KS; ++s) acc[nt] = mfma16(on ? a[x][s] : 0.f, b[x][nt][s], acc[nt]);
        }
      };
      int i0 = 0;
      if constexpr (R <= 64)  // sixteen ids in flight: 288 registers at rank 128
        for (; i0 + 16 <= n; i0 += 16) round(std::integral_constant<int, 16>{}, i0);
      for (; i0 < n; i0 += UB) round(std::integral_constant<int, UB>{}, i0);
    }
    float* dst = dPsum + (size_t)q * PN;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) dst[(4 * kg + v) * R + nt * 16 + l16] = acc[nt][v];
  }
}

// ---------------------------------------------------------------------------------------------
// part3[c]^T = sum over the <= 16 unique ids u of one by-i3 chunk of g_u^T P_q(u)
// (D3 x 16 times 16 x R; the D3 rows occupy the first rows of a 16-row tile), UB ids at a time.
template <int R, int D3, int UB>
__device__ __forceinline__ void dg3_chunk(
    int c, const float* __restrict__ P, const float* __restrict__ grad,
    const float* __restrict__ gsum, const int2* __restrict__ c3_item,
    const int4* __restrict__ c3_desc, float* __restrict__ part3) {
  constexpr int PN = 16 * R, S3 = R * D3, D = 16 * D3, NT = (R + 15) / 16;
  const int lane = threadIdx.x % kWave;
  const int l16 = lane % 16, kg = lane / 16;
  // rank 8: half of the 16 columns of the only tile exist; the others load column 0 and are dropped
  const bool col_on = R >= 16 || l16 < R;
  const int lcol = col_on ? l16 : 0;
  {
    const int2 item = c3_item[(size_t)c * kChunk3 + lane % kChunk3];
    const int cnt = c3_desc[c].z;
    // records past the chunk's count are unwritten; only lanes below cnt are ever read
    const int mycode = item.x, myq = item.y;
    f4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 < cnt; i0 += UB) {
      float a[UB][4], b[UB][NT][4];
#pragma unroll
      for (int x = 0; x < UB; ++x) {
        const int i = min(i0 + x, cnt - 1);
        const float* gp = grad_row_ptr(lane_value(mycode, i), grad, gsum, D) + (4 * kg) * D3 +
                          (l16 < D3 ? l16 : 0);
        const float* pp = P + (size_t)lane_value(myq, i) * PN + (4 * kg) * R + lcol;
#pragma unroll
        for (int s = 0; s < 4; ++s) a[x][s] = gp[s * D3];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int s = 0; s < 4; ++s) b[x][nt][s] = pp[s * R + nt * 16];
      }
      TT_LOADS_DONE();
#pragma unroll
      for (int x = 0; x < UB; ++x) {
        const bool on = (i0 + x < cnt) && (l16 < D3);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int s = 0; s < 4; ++s) acc[nt] = mfma16(on ? a[x][s] : 0.f, b[x][nt][s], acc[nt]);
      }
    }
    float* dst = part3 + (size_t)c * S3;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int j3 = 4 * kg + v;
        if (j3 < D3 && col_on) dst[(nt * 16 + l16) * D3 + j3] = acc[nt][v];
      }
  }
}

// ---------------------------------------------------------------------------------------------
// Value of v in the lane `by` places further on in the same row of 16 lanes (a cross-lane move in
// the vector ALU; lanes whose source falls outside the row get their own value back, and are not
// used).
template <int BY>
__device__ __forceinline__ float row_lane_up(float v) {
  if constexpr (BY == 0) return v;
  else
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v),
                                           0x100 + BY /* row_shl:BY */, 0xf, 0xf, false));
}

// The same partial sum for ranks 64 and 128, where a prefix product is 4 to 8 KiB and the loads
// above would be 16 to 32 four-byte loads per id.  The contraction runs over the 16 rows m = 4*j1 + j2 of the product; lane group kg takes j2 = kg
// and the four j1.  The product comes from its second copy Pt[q][j2][b][j1]: one 16-byte load per
// 16 columns b.  The gradient row (16 x D3, row-major) is read with 4/G loads that together cover
// it contiguously, G = 16/D3: lane l16 = jj*D3 + j3 of group kg reads g[4*(x*G + jj) + kg][j3], and
// the lanes j3 < D3 that feed the matrix cores fetch the values of jj > 0 from their row.
template <int R, int D3, int UB>
__device__ __forceinline__ void dg3_chunk_pt(
    int c, const float* __restrict__ Pt, const float* __restrict__ grad,
    const float* __restrict__ gsum, const int2* __restrict__ c3_item,
    const int4* __restrict__ c3_desc, float* __restrict__ part3) {
  constexpr int PN = 16 * R, S3 = R * D3, D = 16 * D3, NT = (R + 15) / 16;
  constexpr int G = 16 / D3, NL = 4 / G;  // lanes groups per row of 16 lanes; loads per gradient row
  const int lane = threadIdx.x % kWave;
  const int l16 = lane % 16, kg = lane / 16;
  const int j3 = l16 % D3, jj = l16 / D3;
  // rank 8: half of the 16 columns of the only tile exist; the others load column 0 and are dropped
  const bool col_on = R >= 16 || l16 < R;
  const int lcol = col_on ? l16 : 0;
  {
    const int2 item = c3_item[(size_t)c * kChunk3 + lane % kChunk3];
    const int cnt = c3_desc[c].z;
    // records past the chunk's count are unwritten; only lanes below cnt are ever read
    const int mycode = item.x, myq = item.y;
    f4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 < cnt; i0 += UB) {
      float ld[UB][NL];
      f4 b[UB][NT];
#pragma unroll
      for (int x = 0; x < UB; ++x) {
        const int i = min(i0 + x, cnt - 1);
        const float* gp = grad_row_ptr(lane_value(mycode, i), grad, gsum, D) + kg * D3 + j3;
        const float* pp = Pt + (size_t)lane_value(myq, i) * PN + kg * (4 * R) + lcol * 4;
#pragma unroll
        for (int y = 0; y < NL; ++y) ld[x][y] = gp[4 * (y * G + jj) * D3];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[x][nt] = *(const f4*)(pp + nt * 64);
      }
      TT_LOADS_DONE();
#pragma unroll
      for (int x = 0; x < UB; ++x) {
        const bool on = (i0 + x < cnt) && (l16 < D3);
        float a[4];  // a[j1] = g[4*j1 + kg][j3]
#pragma unroll
        for (int y = 0; y < NL; ++y) {
          if constexpr (G == 2) {
            a[2 * y] = ld[x][y];
            a[2 * y + 1] = row_lane_up<8>(ld[x][y]);
          } else {
            a[0] = ld[x][y];
            a[1] = row_lane_up<4>(ld[x][y]);
            a[2] = row_lane_up<8>(ld[x][y]);
            a[3] = row_lane_up<12>(ld[x][y]);
          }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int s = 0; s < 4; ++s) acc[nt] = mfma16(on ? a[s] : 0.f, b[x][nt][s], acc[nt]);
      }
    }
    float* dst = part3 + (size_t)c * S3;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int o3 = 4 * kg + v;
        if (o3 < D3 && col_on) dst[(nt * 16 + l16) * D3 + o3] = acc[nt][v];
      }
  }
}

// chunks wave, wave + nwaves, ... in index order
template <int R, int D3, int UB>
__device__ __forceinline__ void dg3_role(
    int wave, int nwaves, const float* __restrict__ P, const float* __restrict__ grad,
    const float* __restrict__ gsum, const int2* __restrict__ c3_item,
    const int4* __restrict__ c3_desc, float* __restrict__ part3, const Counters* __restrict__ ctr) {
  const int nchunk = ctr->nchunk3;
  for (int c = wave; c < nchunk; c += nwaves)
    dg3_chunk_pt<R, D3, UB>(c, P, grad, gsum, c3_item, c3_desc, part3);
}

// ---------------------------------------------------------------------------------------------
// The two gradient steps that only need the per-id gradient sums run side by side in one launch:
// even blocks form dPsum per prefix, odd blocks the partial G3 gradients per by-i3 chunk.
template <int R, int D3>
__global__ __launch_bounds__(kMThreads) void k_id_bwd_mfma(
    const float* __restrict__ g3, const float* __restrict__ P, const float* __restrict__ grad,
    const float* __restrict__ gsum, const int* __restrict__ u_code, const int* __restrict__ u_i3,
    const int* __restrict__ q_us, const int2* __restrict__ c3_item,
    const int4* __restrict__ c3_desc, float* __restrict__ dPsum, float* __restrict__ part3,
    const Counters* __restrict__ ctr) {
  const int role = blockIdx.x & 1, block = blockIdx.x >> 1, nblocks = gridDim.x >> 1;
  if (role == 0)
    u_bwd_role<R, D3>(block, nblocks, g3, grad, gsum, u_code, u_i3, q_us, dPsum, ctr);
  else
    dg3_role<R, D3, (R >= 128) ? 2 : (R == 64) ? 4 : 8>(block * kMWaves + (int)threadIdx.x / kWave, nblocks * kMWaves,
                                       P, grad, gsum, c3_item, c3_desc, part3, ctr);
}

// ---------------------------------------------------------------------------------------------
// Ranks up to 32: the whole middle of the backward pass in one launch, without dPsum ever leaving
// the chip.  A block of eight wavefronts owns one by-i2 chunk (<= 16 prefixes q, Bm = G2[i2]):
//   (i)   dPsum_q = sum over the ids u of q of g_u G3[i3(u)]^T, each wavefront two prefixes, four
//         ids of each in flight together; results go to an LDS tile of 64 rows
//         (row = 4*prefix + j1) by 4R columns, Bm sits in LDS beside it
//   (ii)  wavefronts 0..3: dg1part[q] = dPsum_q Bm^T for four prefixes each (operands from LDS)
//   (iii) wavefronts 4..7: 32 columns each of part2[c] = sum_q G1[i1(q)]^T dPsum_q
// Blocks past the chunk range take the by-i3 chunks of the G3 gradient (dg3_role), one per
// wavefront; that step only needs the per-id gradient sums and the cached prefix products, so
// both run side by side.
// Rank 16 needs half the LDS, so its blocks have four wavefronts and twice as many fit a compute
// unit: in (i) each takes four prefixes, two ids of each in flight together (the same eight id
// slots per round; tables with many prefixes and few ids per prefix are what these ranks meet, and
// one pass over four prefixes has half the dependent round trips of two passes over two), then
// (ii), then wavefronts 0 and 1 take (iii).
template <int R>
constexpr int mid_waves() { return R >= 32 ? 8 : 4; }
constexpr int kXcds = 8;

template <int R, int D3>
__global__ __launch_bounds__(mid_waves<R>() * kWave, 6) void k_bwd_mid_mfma(
    const float* __restrict__ g1, const float* __restrict__ g2, const float* __restrict__ g3,
    const float* __restrict__ P, const float* __restrict__ grad, const float* __restrict__ gsum,
    const int* __restrict__ u_code, const int* __restrict__ u_i3, const int4* __restrict__ c2_item,
    const int4* __restrict__ c2_desc, const int2* __restrict__ c3_item,
    const int4* __restrict__ c3_desc, const int* __restrict__ c3_order,
    float* __restrict__ dg1part, float* __restrict__ part2, float* __restrict__ part3,
    int chunk_blocks, const Counters* __restrict__ ctr) {
  static_assert(R == 8 || R == 16 || R == 32, "the LDS tiles are sized for ranks up to 32");
  constexpr int W = 4 * R, S1 = 4 * R, S2 = R * W, S3 = R * D3, D = 16 * D3;
  constexpr int TS = W + 4;  // padded row stride of the LDS tiles (keeps 16-byte alignment)
  constexpr int NT16 = (R + 15) / 16, KS = D3 / 4;
  __shared__ __align__(16) float T[64 * TS];
  __shared__ __align__(16) float Bl[R * TS];
  __shared__ int q_of[16], i1_of[16], u0_of[16], u1_of[16];
  constexpr int kMidWaves = mid_waves<R>(), kMidThreads = kMidWaves * kWave;
  const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
  // Blocks past the by-i2 chunk range take the by-i3 chunks, one per wavefront, in the order of
  // the chunks' first prefixes.  Workgroups go to the eight XCDs round robin, so XCD x takes the
  // x-th eighth of that order and walks it front to back: the prefix products a chunk gathers
  // were then just read by its neighbours through the same L2.
  if ((int)blockIdx.x >= chunk_blocks) {
    const int rel = (int)blockIdx.x - chunk_blocks, xcd = (int)blockIdx.x % kXcds;
    const int per_xcd = ((int)gridDim.x - chunk_blocks) / kXcds * kMidWaves;
    const int n = ctr->nchunk3;
    const int lo = (int)((long long)n * xcd / kXcds), hi = (int)((long long)n * (xcd + 1) / kXcds);
    for (int i = lo + rel / kXcds * kMidWaves + w; i < hi; i += per_xcd)
      dg3_chunk<R, D3, 4>(c3_order ? c3_order[i] : i, P, grad, gsum, c3_item, c3_desc, part3);
    return;
  }
  // records, descriptor and chunk count are read together (the grid never exceeds the tables)
  const int c = blockIdx.x;
  const int4 item = c2_item[(size_t)c * kChunk2 + tid % kChunk2];
  const int4 desc = c2_desc[c];
  if (c >= ctr->nchunk2) return;
  const int bin = desc.x, cnt = desc.z;
  const float* Bm = g2 + (size_t)bin * S2;
  if (tid < 16) {
    const bool on = tid < cnt;  // records past the chunk's count are unwritten
    q_of[tid] = on ? item.x : -1;
    i1_of[tid] = on ? item.y : 0;
    u0_of[tid] = on ? item.z : 0;
    u1_of[tid] = on ? item.w : 0;
  }
  for (int i = tid; i < R * W / 4; i += kMidThreads) {
    const f4 v = ((const f4*)Bm)[i];
    *(f4*)&Bl[((i * 4) / W) * TS + (i * 4) % W] = v;
  }
  __syncthreads();

  const int l16 = lane % 16, kg = lane / 16;
  // rank 8: rows / columns 8..15 of the only 16-wide tile do not exist; such lanes read row 0 and
  // their results are dropped
  const bool rank_on = R >= 16 || l16 < R;
  const int lrow = rank_on ? l16 : 0;
  // (i) this wavefront's G prefixes (local numbers G*w .. G*w+G-1; two with eight wavefronts, four
  // with four) in one pass: eight id slots per round, 8/G ids of each prefix.  Lanes 0..7 hold the
  // round's slots: prefix g = lane / UB of the wavefront, id r*UB + lane % UB of its list.
  {
    constexpr int G = 16 / kMidWaves, UB = 8 / G;
    f4 acc[G][NT16];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int nt = 0; nt < NT16; ++nt) acc[g][nt] = f4{0.f, 0.f, 0.f, 0.f};
    int nmax = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) nmax = max(nmax, u1_of[G * w + g] - u0_of[G * w + g]);
    const int myp = G * w + (lane % 8) / UB;  // the prefix of this lane's slot
    const int myu0 = u0_of[myp], myn = u1_of[myp] - myu0;
    const int rounds = (nmax + UB - 1) / UB;
    for (int r = 0; r < rounds; ++r) {
      const int si = r * UB + lane % UB;
      const bool slot_on = lane < 8 && si < myn;
      const int uu = slot_on ? myu0 + si : 0;
      const int mycode = u_code[uu], myi3 = u_i3[uu];
      float a[8][KS], b[8][NT16][KS];
#pragma unroll
      for (int sl = 0; sl < 8; ++sl) {
        const float* gp = grad_row_ptr(lane_value(mycode, sl), grad, gsum, D) + l16 * D3 + KS * kg;
        const float* cp = g3 + (size_t)lane_value(myi3, sl) * S3 + lrow * D3 + KS * kg;
#pragma unroll
        for (int k = 0; k < KS; ++k) a[sl][k] = gp[k];
#pragma unroll
        for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
          for (int k = 0; k < KS; ++k) b[sl][nt][k] = cp[nt * 16 * D3 + k];
      }
      TT_LOADS_DONE();
      const unsigned long long on_mask = __ballot(slot_on);
#pragma unroll
      for (int sl = 0; sl < 8; ++sl) {
        // wavefront-uniform: empty slots cost no matrix-core time
        if ((on_mask >> sl) & 1ull) {
#pragma unroll
          for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
            for (int k = 0; k < KS; ++k)
              acc[sl / UB][nt] = mfma16(a[sl][k], b[sl][nt][k], acc[sl / UB][nt]);
        }
      }
    }
    // accumulator element v of lane (kg, l16) is dPsum_q[m = 4*kg + v][n = nt*16 + l16], i.e. row
    // j1 = kg of the prefix and column j2*R + n with j2 = v
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (rank_on) T[((G * w + g) * 4 + kg) * TS + v * R + nt * 16 + l16] = acc[g][nt][v];
  }
  __syncthreads();

  if (w < 4) {
    // (ii) tile rows 16w .. 16w+15 (prefixes 4w .. 4w+3) times Bm^T, 16 x 16 output tiles; lane
    // group kg contracts over columns [KQ*kg, KQ*kg + KQ)
    constexpr int KQ = W / 4;
    const f4* arow = (const f4*)&T[(16 * w + l16) * TS + KQ * kg];
    f4 acc[NT16];
#pragma unroll
    for (int nt = 0; nt < NT16; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < KQ / 4; ++j) {
      const f4 x = arow[j];
#pragma unroll
      for (int nt = 0; nt < NT16; ++nt) {
        const f4 y = *(const f4*)&Bl[(16 * nt + lrow) * TS + KQ * kg + 4 * j];
        acc[nt] = mfma16(x.x, y.x, acc[nt]);
        acc[nt] = mfma16(x.y, y.y, acc[nt]);
        acc[nt] = mfma16(x.z, y.z, acc[nt]);
        acc[nt] = mfma16(x.w, y.w, acc[nt]);
      }
    }
    // accumulator element v: tile row 4*kg + v = prefix 4w + kg, j1 = v; column n = 16*nt + l16
    const int qv = q_of[4 * w + kg];
    if (qv >= 0) {
#pragma unroll
      for (int nt = 0; nt < NT16; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (rank_on) dg1part[(size_t)qv * S1 + v * R + 16 * nt + l16] = acc[nt][v];
    }
  }
  const int w3 = kMidWaves == 8 ? w - 4 : w;
  if (w3 >= 0 && w3 < W / 32) {
    // (iii) G1 rows of the sixteen prefixes (as the contraction index) times 32 columns of the tile
    const int half = lane / 32, l32 = lane % 32;
    float a[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int ql = 8 * half + j / 4;
      a[j] = g1[(size_t)i1_of[ql] * S1 + (j % 4) * R + (l32 < R ? l32 : 0)];
    }
    TT_LOADS_DONE();
#pragma unroll
    for (int j = 0; j < 32; ++j)
      if (q_of[8 * half + j / 4] < 0 || l32 >= R) a[j] = 0.f;
    const int n = w3 * 32 + l32;
    f16v acc = TT_ZERO16;
#pragma unroll
    for (int j = 0; j < 32; ++j) acc = mfma32(a[j], T[(32 * half + j) * TS + n], acc);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int mrow = 8 * (v / 4) + 4 * half + (v % 4);
      if (mrow < R) part2[(size_t)c * S2 + (size_t)mrow * W + n] = acc[v];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Rows: one wavefront per tile of TSL sorted slots.  The distinct ids of a tile are taken in groups
// of up to 16/D3 consecutive ids that share a prefix: E = P_q (16 x R) times their G3 slices side
// by side (R x 16).  Up to NB = 3 groups are worked on together (operand loads in flight together);
// their rows go through LDS so that one store instruction writes a whole row to every batch
// position that holds the id.  Rows are written with non-temporal stores: nothing on this path
// reads them back.
template <int R, int D3, int TSL>
__global__ __launch_bounds__(kMThreads) void k_row_fwd_mfma(
    int B, const float* __restrict__ g3, const float* __restrict__ P,
    const int4* __restrict__ s_rec, float* __restrict__ out, Counters* ctr) {
  constexpr int PN = 16 * R, S3 = R * D3, D = 16 * D3, UPT = 16 / D3, KQ = R / 4, VPL = D / kWave;
  // groups per batch: 4 cost two wavefronts per SIMD of occupancy; at rank 128 one group's operands
  // are 64 registers already
  constexpr int NB = R >= 128 ? 1 : TSL <= 16 ? 2 : 3;
  __shared__ float ebuf[kMWaves][NB * UPT * D];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int l16 = lane % 16, kg = lane / 16;
  const int ul = l16 / D3, j3 = l16 % D3;
  float* E = ebuf[w];
  const int ntiles = (B + TSL - 1) / TSL;
  for (int tile = blockIdx.x * kMWaves + w; tile < ntiles; tile += gridDim.x * kMWaves) {
    const int s = lane < TSL ? tile * TSL + lane : B;
    const int4 rec = s_rec[min(s, B - 1)];  // {unique-id index, batch position, prefix, i3}
    int mysu = rec.x;
    const uint32_t myb = (uint32_t)rec.y;
    if (s >= B) mysu = -2;  // lanes past the batch: neither an id nor an out-of-range slot
    if (s < B && myb >= (uint32_t)B) atomicOr(&ctr->err, 4);
    // out-of-range ids (the tail of the sorted order) get zero rows
    unsigned long long zero_slots = __ballot(mysu == -1 && myb < (uint32_t)B);
    while (zero_slots) {
      const int sl = __ffsll((long long)zero_slots) - 1;
      zero_slots &= zero_slots - 1;
      float* o = out + (size_t)(uint32_t)lane_value((int)myb, sl) * D + lane * VPL;
#pragma unroll
      for (int e = 0; e < VPL; ++e) o[e] = 0.f;
    }
    const int nv = __popcll(__ballot(mysu >= 0));
    if (nv == 0) continue;
    const int u_lo = lane_value(mysu, 0), nu = lane_value(mysu, nv - 1) - u_lo + 1;
    // lane e takes prefix and i3 of the tile's e-th distinct id from that id's first slot
    int* xch = (int*)E;
    const int su_before = __shfl_up(mysu, 1);
    if (mysu >= 0 && (lane == 0 || mysu != su_before)) {
      xch[mysu - u_lo] = rec.z;
      xch[TSL + mysu - u_lo] = rec.w;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    int myq = xch[min(lane, nu - 1)];
    const int myi3 = xch[TSL + min(lane, nu - 1)];
    if (lane >= nu) myq = -1;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // group starts: every UPT-th id of a run of ids with one prefix
    const int q_before = __shfl_up(myq, 1);
    const unsigned long long run_starts = __ballot(lane < nu && (lane == 0 || myq != q_before));
    const unsigned long long upto = run_starts & (lane == 63 ? ~0ull : ((2ull << lane) - 1ull));
    const int run_first = 63 - __clzll((long long)upto);
    unsigned long long groups = __ballot(lane < nu && ((lane - run_first) % UPT) == 0);
    const int rel = mysu - u_lo;
    while (groups) {
      int st[NB], gsz[NB];
#pragma unroll
      for (int x = 0; x < NB; ++x) {
        if (groups) {
          st[x] = __ffsll((long long)groups) - 1;
          groups &= groups - 1;
          gsz[x] = (groups ? __ffsll((long long)groups) - 1 : nu) - st[x];
        } else {
          st[x] = -1;
          gsz[x] = 0;
        }
      }
      float a[NB][KQ], b[NB][KQ];
      int qx[NB];
#pragma unroll
      for (int x = 0; x < NB; ++x) {
        const int first = st[x] >= 0 ? st[x] : 0;
        const int q = lane_value(myq, first);
        qx[x] = q;
        const int i3 = __shfl(myi3, min(first + ul, nu - 1));
        const float* pc = g3 + (size_t)i3 * S3 + (KQ * kg) * D3 + j3;
        // a group whose prefix is the previous group's takes that group's P operand
        if (x == 0 || q != qx[x - 1]) {
          const float* pf = P + (size_t)(q >= 0 ? q : 0) * PN + l16 * R + KQ * kg;
          if constexpr (KQ % 4 == 0) {
            const f4* pa = (const f4*)pf;
#pragma unroll
            for (int j = 0; j < KQ / 4; ++j) {
              const f4 v = pa[j];
              a[x][4 * j + 0] = v.x;
              a[x][4 * j + 1] = v.y;
              a[x][4 * j + 2] = v.z;
              a[x][4 * j + 3] = v.w;
            }
          } else {  // rank 8: two floats per lane
#pragma unroll
            for (int j = 0; j < KQ; ++j) a[x][j] = pf[j];
          }
        }
#pragma unroll
        for (int j = 0; j < KQ; ++j) b[x][j] = pc[j * D3];
      }
      TT_LOADS_DONE();
#pragma unroll
      for (int x = 1; x < NB; ++x)
        if (qx[x] == qx[x - 1]) {
#pragma unroll
          for (int j = 0; j < KQ; ++j) a[x][j] = a[x - 1][j];
        }
#pragma unroll
      for (int x = 0; x < NB; ++x) {
        f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KQ; ++j) acc = mfma16(a[x][j], b[x][j], acc);
        if (ul < gsz[x]) {
          float* e = E + (st[x] + ul - st[0]) * D + (4 * kg) * D3 + j3;
#pragma unroll
          for (int v = 0; v < 4; ++v) e[v * D3] = acc[v];
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // rows of the ids st[0] .. last of this batch, to every slot that holds them
      int last = st[0] + gsz[0];
#pragma unroll
      for (int x = 1; x < NB; ++x)
        if (st[x] >= 0) last = st[x] + gsz[x];
      for (int k = st[0]; k < last; ++k) {
        float e[VPL];
#pragma unroll
        for (int y = 0; y < VPL; ++y) e[y] = E[(k - st[0]) * D + lane * VPL + y];
        unsigned long long slots = __ballot(rel == k && mysu >= 0);
        while (slots) {
          const int sl = __ffsll((long long)slots) - 1;
          slots &= slots - 1;
          const uint32_t b_row = (uint32_t)lane_value((int)myb, sl);
          if (b_row < (uint32_t)B) stream_store<VPL>(out + (size_t)b_row * D + lane * VPL, e);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Sums grad_out over runs of equal ids (rows of D = 64*VPL floats, VPL floats per lane).
// A block takes 1024 consecutive sorted slots, 64 per wavefront.  Each wavefront loads the rows of
// its slots (32 at a time, all loads in flight together), adds them up run by run in slot order,
// and finishes the runs that lie inside its 64 slots; ids that occur once are skipped, later
// kernels read their row from grad_out directly.  Pieces of runs that cross wavefronts are joined
// in LDS.  No run crosses a block: the index pipeline cuts long runs of one id into entries at
// every multiple of kEntrySlots slots, which is the block size here.
constexpr int kGsumWaves = 16;
constexpr int kGsumThreads = kGsumWaves * kWave;
constexpr int kGsumBlockSlots = kGsumWaves * kWave;  // 1024
static_assert(kGsumBlockSlots == kEntrySlots, "a block must own exactly one entry span");

template <int VPL>
struct LaneVec {
  float v[VPL];
};

// RAGGED: rows of Drt <= 64*VPL floats (any length); lanes past the end of a row carry zeros, and
// rows are read with plain dword loads (their starts need not be 8-byte aligned).
template <int VPL, bool RAGGED = false>
__global__ __launch_bounds__(kGsumThreads) void k_gsum_block(int B, int Drt,
                                                          const float* __restrict__ grad,
                                                          const int* __restrict__ s_u,
                                                          const uint32_t* __restrict__ perm,
                                                          float* __restrict__ gsum, Counters* ctr) {
  constexpr int DP = kWave * VPL;          // padded row length
  const int D = RAGGED ? Drt : DP;
  constexpr int kRows = VPL <= 2 ? 32 : 64 / VPL;  // rows a wavefront has in flight (64 registers)
  __shared__ float part[kGsumWaves][2][DP];  // [wave][0 = head piece, 1 = tail piece]
  __shared__ int head_state[kGsumWaves];    // 0 none, 1 head piece ends in this wave, 2 it runs through
  __shared__ int tail_u[kGsumWaves];        // id whose run starts in this wave and continues, or -1
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int nbt = (B + kGsumBlockSlots - 1) / kGsumBlockSlots;
  for (int bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
    const int wt0 = bt * kGsumBlockSlots + w * kWave;
    const int s = wt0 + lane;
    const int mysu = s < B ? s_u[s] : -1;
    const uint32_t myb = s < B ? perm[s] : 0u;
    if (s < B && myb >= (uint32_t)B) atomicOr(&ctr->err, 8);
    const int prev_su = (wt0 > 0 && wt0 - 1 < B) ? s_u[wt0 - 1] : -2;
    const int next_su = (wt0 + kWave < B) ? s_u[wt0 + kWave] : -2;
    const int nv = __popcll(__ballot(mysu >= 0));
    // a slot needs its row loaded unless its id occurs exactly once in the whole batch
    int su_before = __shfl_up(mysu, 1), su_after = __shfl_down(mysu, 1);
    if (lane == 0) su_before = prev_su;
    if (lane == kWave - 1) su_after = next_su;
    const bool need = mysu >= 0 && myb < (uint32_t)B && (su_before == mysu || su_after == mysu);
    const unsigned long long need_mask = __ballot(need);

    if (lane == 0) {
      head_state[w] = 0;
      tail_u[w] = -1;
    }
    LaneVec<VPL> acc;
    int cur = -2, cur_first = 0;
    auto flush = [&](int end_slot) {  // the run of cur covers tile slots [cur_first, end_slot)
      if (cur < 0) return;
      const bool starts_here = cur_first > 0 || prev_su != cur;
      const bool ends_here = end_slot < kWave || next_su != cur;
      if (starts_here && ends_here) {
        if (end_slot - cur_first > 1) {
          float* o = gsum + (size_t)cur * D + lane * VPL;
#pragma unroll
          for (int x = 0; x < VPL; ++x)
            if (!RAGGED || lane * VPL + x < D) o[x] = acc.v[x];
        }
      } else {
        const int h = starts_here ? 1 : 0;
#pragma unroll
        for (int x = 0; x < VPL; ++x) part[w][h][lane * VPL + x] = acc.v[x];
        if (lane == 0) {
          if (h == 0) head_state[w] = ends_here ? 1 : 2;
          else tail_u[w] = cur;
        }
      }
    };
    for (int half = 0; half < kWave / kRows; ++half) {
      if (half * kRows >= nv) break;
      LaneVec<VPL> r[kRows];
#pragma unroll
      for (int k = 0; k < kRows; ++k) {
        const int slot = half * kRows + k;
        const uint32_t b_row = (uint32_t)lane_value((int)myb, slot);
        if ((need_mask >> slot) & 1ull) {
          if constexpr (RAGGED) {
#pragma unroll
            for (int x = 0; x < VPL; ++x)
              r[k].v[x] = lane * VPL + x < D
                              ? __builtin_nontemporal_load(grad + (size_t)b_row * D + lane * VPL + x)
                              : 0.f;
          } else {
            stream_load<VPL>(grad + (size_t)b_row * D + lane * VPL, r[k].v);
          }
        } else {
#pragma unroll
          for (int x = 0; x < VPL; ++x) r[k].v[x] = 0.f;
        }
      }
#pragma unroll
      for (int k = 0; k < kRows; ++k) {
        const int slot = half * kRows + k;
        if (slot < nv) {
          const int u = lane_value(mysu, slot);
          if (u != cur) {
            flush(slot);
            cur = u;
            cur_first = slot;
#pragma unroll
            for (int x = 0; x < VPL; ++x) acc.v[x] = 0.f;
          }
#pragma unroll
          for (int x = 0; x < VPL; ++x) acc.v[x] += r[k].v[x];
        }
      }
    }
    flush(nv);
    __syncthreads();
    // join the pieces inside the block, in wave order
    // (a) the run that begins in this wave's tail
    if (tail_u[w] >= 0) {
      LaneVec<VPL> t;
#pragma unroll
      for (int x = 0; x < VPL; ++x) t.v[x] = part[w][1][lane * VPL + x];
      bool open = true;
      for (int k = w + 1; k < kGsumWaves && open; ++k) {
        if (head_state[k] == 0) {  // cannot happen for a run that continues; keeps the loop safe
          open = false;
          break;
        }
#pragma unroll
        for (int x = 0; x < VPL; ++x) t.v[x] += part[k][0][lane * VPL + x];
        if (head_state[k] == 1) open = false;
      }
      if (open && lane == 0) atomicOr(&ctr->err, 16);  // a run left the block: entries never do
      float* o = gsum + (size_t)tail_u[w] * D;
#pragma unroll
      for (int x = 0; x < VPL; ++x)
        if (!RAGGED || lane * VPL + x < D) o[lane * VPL + x] = t.v[x];
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// dispatch

bool mfma_shape(const Shape& s) {
  return s.d1 == 4 && s.d2 == 4 && s.r1 == s.r2 &&
         (s.r1 == 8 || s.r1 == 16 || s.r1 == 32 || s.r1 == 64 || s.r1 == 128) &&
         (s.d3 == 4 || s.d3 == 8);
}

static inline int cdivi(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline int grid_cap(int64_t items, int cap) {
  return (int)std::max<int64_t>(1, std::min<int64_t>(items, cap));
}
constexpr int kMGridCap = 256 * 8;

// Blocks of `threads` threads of a kernel that the current device holds at once (what the
// runtime's occupancy calculation says for the kernel's registers and LDS, times the compute
// units).  The per-chunk kernels launch that many blocks at most and walk their work units with
// the grid's stride: every block is resident from the start, none waits for another to end.
template <class K>
static int resident_blocks(K kernel, int threads) {
  int per_cu = 0, dev = 0, cus = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess ||
      per_cu < 1)
    per_cu = 8;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  return per_cu * cus;
}

#define TT_DISPATCH_R(R_, CALL)      \
  switch (R_) {                      \
    case 16: { constexpr int R = 16; CALL; } break; \
    case 32: { constexpr int R = 32; CALL; } break; \
    case 64: { constexpr int R = 64; CALL; } break; \
    default: { constexpr int R = 128; CALL; } break; \
  }
// the kernels that also exist for rank 8 (prefix products and rows; rank 8 takes the fused middle
// kernel in the backward pass)
#define TT_DISPATCH_R8(R_, CALL)                    \
  if ((R_) == 8) {                                  \
    constexpr int R = 8;                            \
    CALL;                                           \
  } else {                                          \
    TT_DISPATCH_R(R_, CALL)                         \
  }
#define TT_DISPATCH_RD(R_, D3_, CALL)                 \
  if ((D3_) == 4) {                                   \
    constexpr int D3 = 4;                             \
    TT_DISPATCH_R(R_, CALL)                           \
  } else {                                            \
    constexpr int D3 = 8;                             \
    TT_DISPATCH_R(R_, CALL)                           \
  }

void launch_prefix_fwd_mfma(const Plan& pl, const Workspace& ws, const float* g1, const float* g2,
                            int B, hipStream_t st) {
  // one block per possible work unit (upper bound from B); blocks past the real count return at once
  const int64_t chunks = cdivi(std::min<int64_t>(B, pl.maxQ), kChunk2) + pl.sh.n2;
  const int units = (int)(chunks * pf_units(pl.sh.r1));
  // Rank 64 launches no more blocks than the device holds at once and lets them walk the units: its
  // batches often have far fewer chunks than their size allows (clustered ids), and the blocks
  // that would find no work cost more to dispatch than the work itself.  The other ranks measured
  // better with one block per possible unit.
  int grid = units;
  if (pl.sh.r1 == 64) {
    if (pl.unit_slots[0] == 0) pl.unit_slots[0] = resident_blocks(k_prefix_fwd_mfma<64>, kWave);
    grid = std::min(units, pl.unit_slots[0]);
  }
  TT_DISPATCH_R8(pl.sh.r1, (k_prefix_fwd_mfma<R><<<grid, kWave, 0, st>>>(
                               g1, g2, ws.c2_item, ws.c2_desc, ws.P, ws.Pt, units, ws.ctr)));
}

void launch_prefix_bwd_mfma(const Plan& pl, const Workspace& ws, const float* g1, const float* g2,
                            int B, hipStream_t st) {
  const int64_t chunks = cdivi(std::min<int64_t>(B, pl.maxQ), kChunk2) + pl.sh.n2;
  const int units = (int)(chunks * pb_units(pl.sh.r1));
  int grid = units;  // as for the forward kernel
  if (pl.sh.r1 == 64) {
    if (pl.unit_slots[1] == 0) pl.unit_slots[1] = resident_blocks(k_prefix_bwd_mfma<64>, kWave);
    grid = std::min(units, pl.unit_slots[1]);
  }
  TT_DISPATCH_R(pl.sh.r1, (k_prefix_bwd_mfma<R><<<grid, kWave, 0, st>>>(
                              g1, g2, ws.dPsum, ws.c2_item, ws.c2_desc, ws.dg1part, ws.part2,
                              units, ws.ctr)));
}

void launch_id_bwd_mfma(const Plan& pl, const Workspace& ws, const float* g3, const float* grad,
                        int B, hipStream_t st) {
  // both roles loop over their work with a stride of half the grid (which must be even)
  const int64_t waves_q = std::min<int64_t>(B, pl.maxQ), waves_c = cdivi(B, chunk3_fill(B)) + (int64_t)pl.sh.n3;
  const int per_role = grid_cap(cdivi(std::max(waves_q, waves_c), kMWaves), kMGridCap);
  TT_DISPATCH_RD(pl.sh.r1, pl.sh.d3, (k_id_bwd_mfma<R, D3><<<2 * per_role, kMThreads, 0, st>>>(
                                         g3, ws.Pt, grad, ws.gsum, ws.u_code, ws.u_i3, ws.q_us,
                                         ws.c3_item, ws.c3_desc, ws.dPsum, ws.part3, ws.ctr)));
}

// true when k_bwd_mid_mfma covers the shape (else: k_id_bwd_mfma followed by k_prefix_bwd_mfma)
bool mfma_fused_mid(const Shape& s) { return mfma_shape(s) && s.r1 <= 32; }

void launch_bwd_mid_mfma(const Plan& pl, const Workspace& ws, const float* g1, const float* g2,
                         const float* g3, const float* grad, int B, hipStream_t st) {
  const int chunk_blocks = cdivi(std::min<int64_t>(B, pl.maxQ), kChunk2) + (int)pl.sh.n2;
  const int waves = pl.sh.r1 <= 16 ? mid_waves<16>() : mid_waves<32>();
  const int* order = (ws.has_order && chunks_ordered(pl, B)) ? ws.c3_order : nullptr;
  // the same number of by-i3 blocks on every XCD
  const int dg3_blocks =
      kXcds * cdivi(cdivi(cdivi(B, chunk3_fill(B)) + (int64_t)pl.sh.n3, kXcds), waves);
#define TT_MID(RR, DD)                                                                            \
  k_bwd_mid_mfma<RR, DD><<<chunk_blocks + dg3_blocks, waves * kWave, 0, st>>>(                    \
      g1, g2, g3, ws.P, grad, ws.gsum, ws.u_code, ws.u_i3, ws.c2_item, ws.c2_desc, ws.c3_item,    \
      ws.c3_desc, order, ws.dg1part, ws.part2, ws.part3, chunk_blocks, ws.ctr)
  if (pl.sh.r1 == 8) {
    if (pl.sh.d3 == 4) TT_MID(8, 4); else TT_MID(8, 8);
  } else if (pl.sh.r1 == 16) {
    if (pl.sh.d3 == 4) TT_MID(16, 4); else TT_MID(16, 8);
  } else {
    if (pl.sh.d3 == 4) TT_MID(32, 4); else TT_MID(32, 8);
  }
#undef TT_MID
}

void launch_row_fwd_mfma(const Plan& pl, const Workspace& ws, const float* g3, int B, float* out,
                         hipStream_t st) {
#define TT_ROW(D3_, TSL_)                                                                        \
  {                                                                                              \
    constexpr int D3 = D3_, TSL = TSL_;                                                          \
    const int grid = grid_cap(cdivi(cdivi(B, TSL), kMWaves), 1 << 20);                           \
    TT_DISPATCH_R8(pl.sh.r1, (k_row_fwd_mfma<R, D3, TSL><<<grid, kMThreads, 0, st>>>(            \
                                 B, g3, ws.P, ws.s_rec, out, ws.ctr)));                          \
  }
  const bool small = B <= kRowSmallBatch;
  if (pl.sh.d3 == 4) {
    if (small) TT_ROW(4, 16) else TT_ROW(4, 32)
  } else {
    if (small) TT_ROW(8, 16) else TT_ROW(8, 32)
  }
#undef TT_ROW
}

void launch_gsum_block(const Plan& pl, const Workspace& ws, const float* grad, int B,
                       hipStream_t st) {
  const int grid = grid_cap(cdivi(B, kGsumBlockSlots), kMGridCap);
  const uint32_t* perm = ws.val[(pl.passes - 1) & 1];
  const int D = pl.sh.D;
  if (D == 64)
    k_gsum_block<1><<<grid, kGsumThreads, 0, st>>>(B, D, grad, ws.s_u, perm, ws.gsum, ws.ctr);
  else if (D == 128)
    k_gsum_block<2><<<grid, kGsumThreads, 0, st>>>(B, D, grad, ws.s_u, perm, ws.gsum, ws.ctr);
  else if (D <= 64)
    k_gsum_block<1, true><<<grid, kGsumThreads, 0, st>>>(B, D, grad, ws.s_u, perm, ws.gsum, ws.ctr);
  else if (D <= 128)
    k_gsum_block<2, true><<<grid, kGsumThreads, 0, st>>>(B, D, grad, ws.s_u, perm, ws.gsum, ws.ctr);
  else
    k_gsum_block<4, true><<<grid, kGsumThreads, 0, st>>>(B, D, grad, ws.s_u, perm, ws.gsum, ws.ctr);
}

// rows this long have a block version of the gradient sums (any shape)
bool gsum_block_rows(const Shape& s) { return s.D <= 4 * kWave; }

}  // namespace ttemb

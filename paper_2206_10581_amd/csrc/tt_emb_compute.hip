// Arithmetic kernels of the TT-embedding path for any table shape (gfx950, fp32; the block products
// run on the matrix cores, the rest on the vector ALUs).
//
// Forward (paper Section 3, the row construction after Eq. "tt-embedding"):
//   P_q = G1[i1] G2[i2]            once per distinct (i1,i2) prefix q, kept for the backward pass
//   E_u = reshape(P_q) G3[i3]      once per run of equal ids inside a tile of sorted slots,
//                                  written to every batch position that holds the id
// Backward (chain rule through the two products) and update (plain SGD):
//   g_u     = sum of grad_out over the positions of unique id u
//   dPsum_q = sum over u in q of g_u G3[i3(u)]^T
//   dG3[i3] = sum over u with that i3 of P_q(u)^T g_u         (chunked partial sums)
//   dG1[i1] = sum over q with that i1 of dPsum_q G2[i2(q)]^T  (one term per q)
//   dG2[i2] = sum over q with that i2 of G1[i1(q)]^T dPsum_q  (chunked partial sums)
//   Gk[s]  -= lr * dGk[s] for touched slices, after every gradient has been formed
// Every sum runs over a list whose order the index pipeline fixed, so results are reproducible
// bit for bit.
#include <algorithm>

#include <hip/hip_ext.h>

#include "tt_emb_internal.h"

namespace ttemb {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;

__device__ __forceinline__ void flag_error(Counters* ctr, int bit) { atomicOr(&ctr->err, bit); }

// Gradient row of unique id u: the batch row itself when the id occurs once, else its sum.
__device__ __forceinline__ const float* grad_of_unique(int u, const int* __restrict__ u_code,
                                                       const float* __restrict__ grad,
                                                       const float* __restrict__ gsum, int D) {
  const int code = u_code[u];
  return code >= 0 ? grad + (size_t)code * D : gsum + (size_t)(-code - 1) * D;
}

// Copies n elements with NT threads (tid = 0..NT-1), eight loads of a thread in flight together:
// a plain `for (e...) dst[e] = src[e]` with a run-time bound waits for every load in turn.
template <int NT, class LD, class ST>
__device__ __forceinline__ void staged_copy(int n, int tid, LD load, ST store) {
  constexpr int kFlight = 8;
  for (int e0 = tid; e0 < n; e0 += kFlight * NT) {
    float v[kFlight];
#pragma unroll
    for (int j = 0; j < kFlight; ++j) {
      const int e = e0 + j * NT;
      v[j] = e < n ? load(e) : 0.f;
    }
#pragma unroll
    for (int j = 0; j < kFlight; ++j) {
      const int e = e0 + j * NT;
      if (e < n) store(e, v[j]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// C(m, n) = sum over k < K of A(m, k) * B(k, n) for m < M, n < N, by one block of kThreads threads:
// 64 x 64 output tiles, the operands staged through LDS sixteen k at a time (zero beyond M, N, K),
// each of the four wavefronts forming a 32 x 32 quadrant with v_mfma_f32_16x16x4f32 (fp32 in, fp32
// accumulate).  fa(m, k), fb(k, n) fetch one operand element, fc(m, n, value) takes one result; the
// *_KFAST flags say which index neighbouring threads should vary while staging (the one that is
// contiguous in memory).  The order of every sum is fixed by M, N, K alone.  All threads of the
// block must call it with the same M, N, K.
constexpr int kGemmTile = 64, kGemmDepth = 16;
constexpr int kGemmStride = kGemmTile + 16;  // row stride 16 mod 32 banks: the four k of an MFMA
                                             // operand read land on disjoint bank halves
struct GemmLds {
  float a[kGemmDepth][kGemmStride];
  float b[kGemmDepth][kGemmStride];
};
typedef float gemm_f4 __attribute__((ext_vector_type(4)));

template <bool A_KFAST, bool B_KFAST, class FA, class FB, class FC>
__device__ __forceinline__ void block_gemm(GemmLds& L, int M, int N, int K, FA fa, FB fb, FC fc) {
  static_assert(kThreads == 256, "four wavefronts, one 32 x 32 quadrant each");
  constexpr int kPer = kGemmTile * kGemmDepth / kThreads;  // operand elements a thread stages
  const int t = threadIdx.x, w = t / kWave, lane = t % kWave;
  const int l16 = lane % 16, kg = lane / 16;
  const int wm = (w / 2) * 32, wn = (w % 2) * 32;
  for (int m0 = 0; m0 < M; m0 += kGemmTile)
    for (int n0 = 0; n0 < N; n0 += kGemmTile) {
      gemm_f4 acc[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = gemm_f4{0.f, 0.f, 0.f, 0.f};
      // the operands of step k0 + kGemmDepth are fetched while step k0 is multiplied
      float ra[kPer], rb[kPer];
      auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
          const int e = t + i * kThreads;
          const int ak = A_KFAST ? e % kGemmDepth : e / kGemmTile;
          const int am = A_KFAST ? e / kGemmDepth : e % kGemmTile;
          ra[i] = (m0 + am < M && k0 + ak < K) ? fa(m0 + am, k0 + ak) : 0.f;
          const int bk = B_KFAST ? e % kGemmDepth : e / kGemmTile;
          const int bn = B_KFAST ? e / kGemmDepth : e % kGemmTile;
          rb[i] = (n0 + bn < N && k0 + bk < K) ? fb(k0 + bk, n0 + bn) : 0.f;
        }
      };
      fetch(0);
      // quadrants that lie entirely beyond M or N have nothing to multiply (wavefront-uniform)
      const bool live = m0 + wm < M && n0 + wn < N;
      for (int k0 = 0; k0 < K; k0 += kGemmDepth) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
          const int e = t + i * kThreads;
          L.a[A_KFAST ? e % kGemmDepth : e / kGemmTile][A_KFAST ? e / kGemmDepth : e % kGemmTile] = ra[i];
          L.b[B_KFAST ? e % kGemmDepth : e / kGemmTile][B_KFAST ? e / kGemmDepth : e % kGemmTile] = rb[i];
        }
        __syncthreads();
        if (k0 + kGemmDepth < K) fetch(k0 + kGemmDepth);
        if (live) {
#pragma unroll
          for (int ks = 0; ks < kGemmDepth / 4; ++ks) {
            // operand layouts of the instruction: A[i][k] in lane 16*k + i, B[k][j] in lane 16*k + j
            const float a0 = L.a[4 * ks + kg][wm + l16], a1 = L.a[4 * ks + kg][wm + 16 + l16];
            const float b0 = L.b[4 * ks + kg][wn + l16], b1 = L.b[4 * ks + kg][wn + 16 + l16];
            acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc[1][1], 0, 0, 0);
          }
        }
        __syncthreads();
      }
      // accumulator element v of lane (kg, l16) is C[4*kg + v][l16] of its 16 x 16 tile
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int m = m0 + wm + 16 * i + 4 * kg + v, n = n0 + wn + 16 * j + l16;
            if (m < M && n < N) fc(m, n, acc[i][j][v]);
          }
    }
}

// The same product by one wavefront alone (32 x 32 output tiles, LDS of its own, no block barrier):
// for many small products it keeps all four wavefronts of a block busy on different ones.
constexpr int kWaveTile = 32;
constexpr int kWaveStride = kWaveTile + 16;
struct WaveGemmLds {
  float a[kGemmDepth][kWaveStride];
  float b[kGemmDepth][kWaveStride];
};

template <bool A_KFAST, bool B_KFAST, class FA, class FB, class FC>
__device__ __forceinline__ void wave_gemm(WaveGemmLds& L, int M, int N, int K, FA fa, FB fb, FC fc) {
  constexpr int kPer = kWaveTile * kGemmDepth / kWave;  // operand elements a lane stages
  const int lane = threadIdx.x % kWave, l16 = lane % 16, kg = lane / 16;
  for (int m0 = 0; m0 < M; m0 += kWaveTile)
    for (int n0 = 0; n0 < N; n0 += kWaveTile) {
      gemm_f4 acc[2][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = gemm_f4{0.f, 0.f, 0.f, 0.f};
      for (int k0 = 0; k0 < K; k0 += kGemmDepth) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
          const int e = lane + i * kWave;
          const int ak = A_KFAST ? e % kGemmDepth : e / kWaveTile;
          const int am = A_KFAST ? e / kGemmDepth : e % kWaveTile;
          L.a[ak][am] = (m0 + am < M && k0 + ak < K) ? fa(m0 + am, k0 + ak) : 0.f;
          const int bk = B_KFAST ? e % kGemmDepth : e / kWaveTile;
          const int bn = B_KFAST ? e / kGemmDepth : e % kWaveTile;
          L.b[bk][bn] = (n0 + bn < N && k0 + bk < K) ? fb(k0 + bk, n0 + bn) : 0.f;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int ks = 0; ks < kGemmDepth / 4; ++ks) {
          const float a0 = L.a[4 * ks + kg][l16], a1 = L.a[4 * ks + kg][16 + l16];
          const float b0 = L.b[4 * ks + kg][l16], b1 = L.b[4 * ks + kg][16 + l16];
          acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[0][0], 0, 0, 0);
          acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b1, acc[0][1], 0, 0, 0);
          acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b0, acc[1][0], 0, 0, 0);
          acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int m = m0 + 16 * i + 4 * kg + v, n = n0 + 16 * j + l16;
            if (m < M && n < N) fc(m, n, acc[i][j][v]);
          }
    }
}

// ---------------------------------------------------------------------------------------------
// forward

// P_q = A * Bm, A = G1[i1] (d1 x r1), Bm = G2[i2] (r1 x d2*r2), for the <= 16 prefixes of one
// by-i2 chunk at a time: their A stacked are the rows of one product with the shared Bm.
__global__ __launch_bounds__(kThreads) void k_prefix_fwd(Shape sh, const float* __restrict__ g1,
                                                         const float* __restrict__ g2,
                                                         const int4* __restrict__ c2_desc,
                                                         const int4* __restrict__ c2_item,
                                                         float* __restrict__ P,
                                                         const Counters* __restrict__ ctr) {
  __shared__ GemmLds L;
  __shared__ int q_of[kChunk2], i1_of[kChunk2];
  const int nchunk = ctr->nchunk2;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int4 desc = c2_desc[c];
    const int cnt = desc.z;
    __syncthreads();  // the previous chunk's readers of q_of / i1_of are done
    if ((int)threadIdx.x < cnt) {
      const int4 it = c2_item[(size_t)c * kChunk2 + threadIdx.x];
      q_of[threadIdx.x] = it.x;
      i1_of[threadIdx.x] = it.y;
    }
    __syncthreads();
    const float* Bm = g2 + (size_t)desc.x * sh.S2;
    block_gemm<true, false>(
        L, cnt * sh.d1, sh.W, sh.r1,
        [&](int m, int k) { return g1[(size_t)i1_of[m / sh.d1] * sh.S1 + (m % sh.d1) * sh.r1 + k]; },
        [&](int k, int n) { return Bm[(size_t)k * sh.W + n]; },
        [&](int m, int n, float v) { P[(size_t)q_of[m / sh.d1] * sh.PN + (m % sh.d1) * sh.W + n] = v; });
  }
}

// One wavefront per tile of kTileSlots sorted slots: E = reshape(P_q) * G3[i3] when the id changes,
// then one row store per slot.  Out-of-range ids get zero rows.
__global__ __launch_bounds__(kThreads) void k_row_fwd(Shape sh, int B, const float* __restrict__ g3,
                                                      const float* __restrict__ P,
                                                      const int* __restrict__ s_u,
                                                      const uint32_t* __restrict__ perm,
                                                      const int* __restrict__ u_i3,
                                                      const int* __restrict__ u_q,
                                                      float* __restrict__ out, Counters* ctr) {
  extern __shared__ float lds[];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  float* E = lds + (size_t)w * sh.D;
  const int ntiles = (B + kTileSlots - 1) / kTileSlots;
  for (int tile = blockIdx.x * kWavesPerBlock + w; tile < ntiles;
       tile += gridDim.x * kWavesPerBlock) {
    const int s1 = min((tile + 1) * kTileSlots, B);
    int cur = -2;
    for (int s = tile * kTileSlots; s < s1; ++s) {
      const int u = s_u[s];
      const uint32_t b = perm[s];
      if (b >= (uint32_t)B) {
        flag_error(ctr, 1);
        continue;
      }
      float* o = out + (size_t)b * sh.D;
      if (u < 0) {
        for (int e = lane; e < sh.D; e += kWave) o[e] = 0.f;
        continue;
      }
      if (u != cur) {
        cur = u;
        const float* Pq = P + (size_t)u_q[u] * sh.PN;
        const float* C = g3 + (size_t)u_i3[u] * sh.S3;
        for (int e = lane; e < sh.D; e += kWave) {
          const int m = e / sh.d3, j3 = e % sh.d3;
          float acc = 0.f;
          for (int c = 0; c < sh.r2; ++c) acc = fmaf(Pq[m * sh.r2 + c], C[c * sh.d3 + j3], acc);
          E[e] = acc;
        }
      }
      for (int e = lane; e < sh.D; e += kWave) o[e] = E[e];
    }
  }
}

// The same with the operands staged, and the work cut so that no wavefront has a long chain of
// dependent steps.  Three kinds of job share the launch, one wavefront each:
//   * a distinct id (entry) with at most kTileSlots positions: the wavefront copies P_q (rows padded
//     by one float against bank conflicts) and G3[i3] into LDS of its own, forms E from there and
//     stores it to all positions of the id - the tail of a batch whose ids all differ costs one
//     round trip per wavefront, not one per slot of a tile in turn;
//   * a tile of kTileSlots sorted slots, for the slots of longer entries only (a tile meets at
//     most two of those): E is formed again per tile, so a hot id's thousand stores are spread
//     over thirty wavefronts;
//   * a tile of out-of-range slots (zero rows).
// Needs D + M*(r2+1) + S3 floats of LDS per wavefront (blocks have as many wavefronts, up to four,
// as the budget allows); shapes too large for even one take k_row_fwd.
__global__ __launch_bounds__(kThreads) void k_row_fwd_staged(
    Shape sh, int B, const float* __restrict__ g3, const float* __restrict__ P,
    const int* __restrict__ s_u, const uint32_t* __restrict__ perm, const int* __restrict__ u_rs,
    const int* __restrict__ u_i3, const int* __restrict__ u_q, float* __restrict__ out,
    Counters* ctr) {
  extern __shared__ float lds[];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int ps = sh.r2 + 1;
  float* E = lds + (size_t)w * (sh.D + sh.M * ps + sh.S3);
  float* Pl = E + sh.D;
  float* Cl = Pl + sh.M * ps;
  const int U = ctr->U, nvalid = ctr->nvalid;
  const int long_tiles = (nvalid + kTileSlots - 1) / kTileSlots;
  const int zero_tiles = (B - nvalid + kTileSlots - 1) / kTileSlots;
  const int wpb = (int)blockDim.x / kWave;  // fewer wavefronts per block when the operands are large
  const int stride = gridDim.x * wpb;
  // E = reshape(P_q) * G3[i3] of entry u, left in LDS
  auto form_row = [&](int u) {
    const float* Pq = P + (size_t)u_q[u] * sh.PN;
    const float* C = g3 + (size_t)u_i3[u] * sh.S3;
    for (int e = lane; e < sh.PN; e += kWave) Pl[(e / sh.r2) * ps + e % sh.r2] = Pq[e];
    for (int e = lane; e < sh.S3; e += kWave) Cl[e] = C[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int e = lane; e < sh.D; e += kWave) {
      const float* pr = Pl + (e / sh.d3) * ps;
      const float* cc = Cl + e % sh.d3;
      float acc = 0.f;
      for (int c = 0; c < sh.r2; ++c) acc = fmaf(pr[c], cc[c * sh.d3], acc);
      E[e] = acc;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  // E to the batch positions of slots [s0, s1), at most a wavefront's worth
  auto store_rows = [&](int s0, int s1) {
    const int n = s1 - s0;
    const uint32_t myb = lane < n ? perm[s0 + lane] : 0u;
    for (int k = 0; k < n; ++k) {
      const uint32_t b = (uint32_t)__shfl((int)myb, k);
      if (b >= (uint32_t)B) {
        flag_error(ctr, 1);
        continue;
      }
      float* o = out + (size_t)b * sh.D;
      for (int e = lane; e < sh.D; e += kWave) o[e] = E[e];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  for (int job = blockIdx.x * wpb + w; job < U + long_tiles + zero_tiles; job += stride) {
    if (job < U) {
      const int rs = u_rs[job], re = u_rs[job + 1];
      if (re - rs > kTileSlots) continue;  // its tiles take it
      form_row(job);
      store_rows(rs, re);
    } else if (job < U + long_tiles) {
      const int t0 = (job - U) * kTileSlots, t1 = min(t0 + kTileSlots, nvalid);
      // every lane looks at one slot; the long entries that begin or continue here are found with
      // one ballot (two dependent loads for the whole tile, not two per entry)
      const bool in = lane < kTileSlots && t0 + lane < t1;
      const int mysu = in ? s_u[t0 + lane] : -1;
      const int my_rs = in ? u_rs[mysu] : 0, my_re = in ? u_rs[mysu + 1] : 0;
      const int before = __shfl_up(mysu, 1);
      unsigned long long starts =
          __ballot(in && my_re - my_rs > kTileSlots && (lane == 0 || mysu != before));
      while (starts) {
        const int k = __ffsll((long long)starts) - 1;
        starts &= starts - 1;
        form_row(__shfl(mysu, k));
        store_rows(t0 + k, min(__shfl(my_re, k), t1));
      }
    } else {
      const int s0 = nvalid + (job - U - long_tiles) * kTileSlots, s1 = min(s0 + kTileSlots, B);
      for (int e = lane; e < sh.D; e += kWave) E[e] = 0.f;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      store_rows(s0, s1);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// backward

// Sums grad_out over runs of equal ids, one wavefront per tile of sorted slots.  A run inside one
// tile is finished here; a run that crosses tiles leaves one partial per tile in carry[tile][h]
// (h = 0: the run began in an earlier tile, h = 1: it begins here and continues).
__global__ __launch_bounds__(kThreads) void k_gsum(Shape sh, int B, const float* __restrict__ grad,
                                                   const int* __restrict__ s_u,
                                                   const uint32_t* __restrict__ perm,
                                                   const int* __restrict__ u_rs,
                                                   float* __restrict__ gsum,
                                                   float* __restrict__ carry, Counters* ctr) {
  extern __shared__ float lds[];
  const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  float* acc = lds + (size_t)w * sh.D;
  const int D = sh.D;
  const int ntiles = (B + kTileSlots - 1) / kTileSlots;
  for (int tile = blockIdx.x * kWavesPerBlock + w; tile < ntiles;
       tile += gridDim.x * kWavesPerBlock) {
    const int t0 = tile * kTileSlots, t1 = t0 + kTileSlots;
    const int s1 = min(t1, B);
    int cur = -2;  // no run open (-1 is the marker of an out-of-range slot)
    for (int s = t0; s <= s1; ++s) {
      const int u = (s < s1) ? s_u[s] : -1;
      if (u != cur) {
        if (cur >= 0) {  // close the run of cur
          const int rs = u_rs[cur], re = u_rs[cur + 1];
          if (rs >= t0 && re <= t1) {
            if (re - rs > 1)
              for (int e = lane; e < D; e += kWave) gsum[(size_t)cur * D + e] = acc[e];
          } else {
            float* c = carry + ((size_t)tile * 2 + (rs < t0 ? 0 : 1)) * D;
            for (int e = lane; e < D; e += kWave) c[e] = acc[e];
          }
        }
        if (u < 0) break;  // out-of-range ids fill the tail of the sorted order
        cur = u;
        for (int e = lane; e < D; e += kWave) acc[e] = 0.f;
      }
      const uint32_t b = perm[s];
      if (b >= (uint32_t)B) {
        flag_error(ctr, 2);
        continue;
      }
      const float* g = grad + (size_t)b * D;
      for (int e = lane; e < D; e += kWave) acc[e] += g[e];
    }
  }
}

// Finishes the runs that cross tiles: the tile in which such a run begins adds up its partials in
// tile order.
__global__ __launch_bounds__(kThreads) void k_gsum_fix(Shape sh, const int* __restrict__ s_u,
                                                       const int* __restrict__ u_rs,
                                                       const float* __restrict__ carry,
                                                       float* __restrict__ gsum,
                                                       const Counters* __restrict__ ctr) {
  const int nvalid = ctr->nvalid, D = sh.D;
  const int ntiles = (nvalid + kTileSlots - 1) / kTileSlots;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int t0 = tile * kTileSlots, t1 = t0 + kTileSlots;
    const int u = s_u[min(t1, nvalid) - 1];
    const int rs = u_rs[u], re = u_rs[u + 1];
    if (rs < t0 || re <= t1) continue;
    const int tl = (re - 1) / kTileSlots;
    for (int e = threadIdx.x; e < D; e += kThreads) {
      float a = carry[((size_t)tile * 2 + 1) * D + e];
      for (int t = tile + 1; t <= tl; ++t) a += carry[((size_t)t * 2) * D + e];
      gsum[(size_t)u * D + e] = a;
    }
  }
}

// dPsum_q = sum over the unique ids u of prefix q of g_u * G3[i3(u)]^T, g_u read as (d1*d2) x d3:
// one product per prefix whose contraction index runs over (u, j3), one wavefront per prefix.
__global__ __launch_bounds__(kThreads) void k_u_bwd(Shape sh, const float* __restrict__ g3,
                                                    const float* __restrict__ grad,
                                                    const float* __restrict__ gsum,
                                                    const int* __restrict__ u_code,
                                                    const int* __restrict__ u_i3,
                                                    const int* __restrict__ q_us,
                                                    float* __restrict__ dPsum,
                                                    const Counters* __restrict__ ctr) {
  __shared__ WaveGemmLds L[kWavesPerBlock];
  const int Q = ctr->Q, w = threadIdx.x / kWave;
  for (int q = blockIdx.x * kWavesPerBlock + w; q < Q; q += gridDim.x * kWavesPerBlock) {
    const int u0 = q_us[q], u1 = q_us[q + 1];
    float* dst = dPsum + (size_t)q * sh.PN;
    wave_gemm<true, true>(
        L[w], sh.M, sh.r2, (u1 - u0) * sh.d3,
        [&](int m, int k) {
          return grad_of_unique(u0 + k / sh.d3, u_code, grad, gsum, sh.D)[m * sh.d3 + k % sh.d3];
        },
        [&](int k, int n) { return g3[(size_t)u_i3[u0 + k / sh.d3] * sh.S3 + n * sh.d3 + k % sh.d3]; },
        [&](int m, int n, float v) { dst[m * sh.r2 + n] = v; });
  }
}

// part3[c] = sum over the unique ids u of chunk c (all with one i3) of P_q(u)^T g_u   (r2 x d3):
// one product per chunk whose contraction index runs over (u, row of P).
__global__ __launch_bounds__(kThreads) void k_dg3(Shape sh, const float* __restrict__ P,
                                                  const float* __restrict__ grad,
                                                  const float* __restrict__ gsum,
                                                  const int2* __restrict__ c3_item,
                                                  const int4* __restrict__ c3_desc,
                                                  float* __restrict__ part3,
                                                  const Counters* __restrict__ ctr) {
  __shared__ GemmLds L;
  __shared__ const float* g_of[kChunk3];
  __shared__ const float* p_of[kChunk3];
  const int nchunk = ctr->nchunk3;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int cnt = c3_desc[c].z;
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
      const int2 it = c3_item[(size_t)c * kChunk3 + threadIdx.x];  // {gradient-row code, prefix}
      g_of[threadIdx.x] = it.x >= 0 ? grad + (size_t)it.x * sh.D : gsum + (size_t)(-it.x - 1) * sh.D;
      p_of[threadIdx.x] = P + (size_t)it.y * sh.PN;
    }
    __syncthreads();
    float* dst = part3 + (size_t)c * sh.S3;
    block_gemm<false, false>(
        L, sh.r2, sh.d3, cnt * sh.M,
        [&](int m, int k) { return p_of[k / sh.M][(k % sh.M) * sh.r2 + m]; },
        [&](int k, int n) { return g_of[k / sh.M][(k % sh.M) * sh.d3 + n]; },
        [&](int m, int n, float v) { dst[m * sh.d3 + n] = v; });
  }
}

// The same for shapes whose P_q and gradient row fit the LDS a few ids at a time: the output is
// small (r2 x d3) and the contraction long, so each thread keeps its outputs and the block walks
// the ids of the chunk, `group` of them per LDS fill, in list order.
__global__ __launch_bounds__(kThreads) void k_dg3_staged(Shape sh, int group,
                                                         const float* __restrict__ P,
                                                         const float* __restrict__ grad,
                                                         const float* __restrict__ gsum,
                                                         const int2* __restrict__ c3_item,
                                                         const int4* __restrict__ c3_desc,
                                                         float* __restrict__ part3,
                                                         const Counters* __restrict__ ctr) {
  extern __shared__ float lds[];  // group * (PN + D) floats
  __shared__ const float* g_of[kChunk3];
  __shared__ const float* p_of[kChunk3];
  constexpr int kOut = 4;  // outputs per thread per pass
  const int nchunk = ctr->nchunk3;
  const int per = sh.PN + sh.D;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int cnt = c3_desc[c].z;
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
      const int2 it = c3_item[(size_t)c * kChunk3 + threadIdx.x];
      g_of[threadIdx.x] = it.x >= 0 ? grad + (size_t)it.x * sh.D : gsum + (size_t)(-it.x - 1) * sh.D;
      p_of[threadIdx.x] = P + (size_t)it.y * sh.PN;
    }
    __syncthreads();
    float* dst = part3 + (size_t)c * sh.S3;
    for (int o0 = 0; o0 < sh.S3; o0 += kThreads * kOut) {
      float acc[kOut];
#pragma unroll
      for (int x = 0; x < kOut; ++x) acc[x] = 0.f;
      for (int t0 = 0; t0 < cnt; t0 += group) {
        const int nt = min(group, cnt - t0);
        __syncthreads();  // the previous fill has been used
        // the fill as one copy of nt * (PN + D) floats: the loads of all its ids overlap
        staged_copy<kThreads>(
            nt * per, (int)threadIdx.x,
            [&](int f) {
              const int t = f / per, e = f % per;
              return e < sh.PN ? p_of[t0 + t][e] : g_of[t0 + t][e - sh.PN];
            },
            [&](int f, float v) { lds[f] = v; });
        __syncthreads();
#pragma unroll
        for (int x = 0; x < kOut; ++x) {
          const int o = o0 + x * kThreads + (int)threadIdx.x;
          if (o < sh.S3) {
            const int b = o / sh.d3, j3 = o % sh.d3;
            for (int t = 0; t < nt; ++t) {
              const float* pl = lds + (size_t)t * per + b;
              const float* gl = lds + (size_t)t * per + sh.PN + j3;
              for (int m = 0; m < sh.M; ++m) acc[x] = fmaf(pl[m * sh.r2], gl[m * sh.d3], acc[x]);
            }
          }
        }
      }
#pragma unroll
      for (int x = 0; x < kOut; ++x) {
        const int o = o0 + x * kThreads + (int)threadIdx.x;
        if (o < sh.S3) dst[o] = acc[x];
      }
    }
  }
}

// For the prefixes q of chunk c (all with one i2, Bm = G2[i2]):
//   dg1part[q] = dPsum_q * Bm^T                      (d1 x r1), the prefixes stacked: one product
//   part2[c]   = sum over q of G1[i1(q)]^T * dPsum_q  (r1 x d2*r2), contraction over (q, j1)
__global__ __launch_bounds__(kThreads) void k_prefix_bwd(Shape sh, const float* __restrict__ g1,
                                                         const float* __restrict__ g2,
                                                         const float* __restrict__ dPsum,
                                                         const int4* __restrict__ c2_desc,
                                                         const int4* __restrict__ c2_item,
                                                         float* __restrict__ dg1part,
                                                         float* __restrict__ part2,
                                                         const Counters* __restrict__ ctr) {
  __shared__ GemmLds L;
  __shared__ int q_of[kChunk2], i1_of[kChunk2];
  const int nchunk = ctr->nchunk2;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int4 desc = c2_desc[c];
    const int cnt = desc.z;
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
      const int4 it = c2_item[(size_t)c * kChunk2 + threadIdx.x];
      q_of[threadIdx.x] = it.x;
      i1_of[threadIdx.x] = it.y;
    }
    __syncthreads();
    const float* Bm = g2 + (size_t)desc.x * sh.S2;
    block_gemm<true, true>(
        L, cnt * sh.d1, sh.r1, sh.W,
        [&](int m, int k) { return dPsum[(size_t)q_of[m / sh.d1] * sh.PN + (m % sh.d1) * sh.W + k]; },
        [&](int k, int n) { return Bm[(size_t)n * sh.W + k]; },
        [&](int m, int n, float v) {
          dg1part[(size_t)q_of[m / sh.d1] * sh.S1 + (m % sh.d1) * sh.r1 + n] = v;
        });
    float* dst = part2 + (size_t)c * sh.S2;
    block_gemm<false, false>(
        L, sh.r1, sh.W, cnt * sh.d1,
        [&](int m, int k) { return g1[(size_t)i1_of[k / sh.d1] * sh.S1 + (k % sh.d1) * sh.r1 + m]; },
        [&](int k, int n) { return dPsum[(size_t)q_of[k / sh.d1] * sh.PN + (k % sh.d1) * sh.W + n]; },
        [&](int m, int n, float v) { dst[(size_t)m * sh.W + n] = v; });
  }
}

// Adds up the partial gradients of every touched slice and applies the update: the SGD step, the
// Adagrad step  S += dG^2,  G -= lr * dG / (sqrt(S) + eps),  or the Adam step
// m = b1 m + (1-b1) dG,  v = b2 v + (1-b2) dG^2,  G -= lr * (m corr1) / (sqrt(v corr2) + eps)
// on the same entries (moments of untouched slices are left alone).
// A job owns up to 256*VEC consecutive entries of one slice (VEC = 4 when slice sizes allow 16-byte
// accesses, else 1).  Its threads are arranged as `parts` groups side by side on the entries; the
// job's list of partials (chunks for G3 and G2, prefixes for G1) is dealt round-robin to the
// groups, whose sums are then added in group order.  parts depends on the slice size only and
// every group walks its share in list order, so the order of each sum is fixed by the list length.
// Jobs: n3*cdiv(S3, span) for G3, then n2*cdiv(S2, span) for G2, then n1*cdiv(S1, span) for G1.
template <int VEC, int RULE>
__global__ __launch_bounds__(kThreads) void k_sgd(Shape sh, float lr, UpdateRule ada,
                                                  float* __restrict__ g1,
                                                  float* __restrict__ g2, float* __restrict__ g3,
                                                  const float* __restrict__ part3,
                                                  const int* __restrict__ c3_start,
                                                  const float* __restrict__ part2,
                                                  const int* __restrict__ c2_start,
                                                  const float* __restrict__ dg1part,
                                                  const int* __restrict__ g1_first,
                                                  const int* __restrict__ g1_end,
                                                  Counters* __restrict__ ctr) {
  constexpr int kSpan = kThreads * VEC, kUnroll = 8;
  __shared__ float red[kThreads][VEC];
  const int sp3 = (sh.S3 + kSpan - 1) / kSpan, sp2 = (sh.S2 + kSpan - 1) / kSpan,
            sp1 = (sh.S1 + kSpan - 1) / kSpan;
  const int64_t jobs3 = (int64_t)sh.n3 * sp3, jobs2 = (int64_t)sh.n2 * sp2,
                jobs1 = (int64_t)sh.n1 * sp1;
  for (int64_t job = blockIdx.x; job < jobs3 + jobs2 + jobs1; job += gridDim.x) {
    const float* src;  // partial k of the list lives at src + k*S
    float* G;
    float* St = nullptr;  // state of the slice: Adagrad sums or Adam first moments
    float* Vt = nullptr;  // Adam second moments
    constexpr bool ADA = RULE != kUpdateSgd, ADAM = RULE == kUpdateAdam;
    int l0, l1, o0, S;
    if (job < jobs3) {
      const int bin = (int)(job / sp3);
      o0 = (int)(job % sp3) * kSpan;
      l0 = c3_start[bin];
      l1 = c3_start[bin + 1];
      src = part3;
      S = sh.S3;
      G = g3 + (size_t)bin * sh.S3;
      if (ADA) St = ada.s3 + (size_t)bin * sh.S3;
      if (ADAM) Vt = ada.v3 + (size_t)bin * sh.S3;
    } else if (job < jobs3 + jobs2) {
      const int64_t j = job - jobs3;
      const int bin = (int)(j / sp2);
      o0 = (int)(j % sp2) * kSpan;
      l0 = c2_start[bin];
      l1 = c2_start[bin + 1];
      src = part2;
      S = sh.S2;
      G = g2 + (size_t)bin * sh.S2;
      if (ADA) St = ada.s2 + (size_t)bin * sh.S2;
      if (ADAM) Vt = ada.v2 + (size_t)bin * sh.S2;
    } else {
      const int64_t j = job - jobs3 - jobs2;
      const int i1 = (int)(j / sp1);
      o0 = (int)(j % sp1) * kSpan;
      l0 = g1_first[i1];
      l1 = g1_end[i1];
      src = dg1part;
      S = sh.S1;
      G = g1 + (size_t)i1 * sh.S1;
      if (ADA) St = ada.s1 + (size_t)i1 * sh.S1;
      if (ADAM) Vt = ada.v1 + (size_t)i1 * sh.S1;
    }
    if (l1 == l0) continue;  // slice not touched by this batch (uniform for the block)
    // thread layout: `lanes` threads side by side cover the job's entries, `parts` such groups
    const int cols = min(kSpan, S - o0);
    int lanes = 1;
    while (lanes * VEC < cols) lanes <<= 1;  // power of two, at most kThreads
    const int parts = kThreads / lanes;
    const int lane = threadIdx.x % lanes, part = threadIdx.x / lanes;
    const bool active = lane * VEC < cols;
    const int o = o0 + (active ? lane * VEC : 0);
    float g_old[VEC], acc[VEC];
#pragma unroll
    for (int x = 0; x < VEC; ++x) {
      g_old[x] = G[o + x];
      acc[x] = 0.f;
    }
    const float* p = src + o;
    int k = l0 + part;
    for (; k + (kUnroll - 1) * parts < l1; k += kUnroll * parts) {
      float v[kUnroll][VEC];
#pragma unroll
      for (int j = 0; j < kUnroll; ++j)
#pragma unroll
        for (int x = 0; x < VEC; ++x) v[j][x] = p[(size_t)(k + j * parts) * S + x];
      __builtin_amdgcn_sched_barrier(0);  // all loads of the round are in flight together
#pragma unroll
      for (int j = 0; j < kUnroll; ++j)
#pragma unroll
        for (int x = 0; x < VEC; ++x) acc[x] += v[j][x];
    }
    for (; k < l1; k += parts)
#pragma unroll
      for (int x = 0; x < VEC; ++x) acc[x] += p[(size_t)k * S + x];
    if (parts > 1) {
#pragma unroll
      for (int x = 0; x < VEC; ++x) red[threadIdx.x][x] = acc[x];
      __syncthreads();
      if (part == 0) {
        for (int q = 1; q < parts; ++q)
#pragma unroll
          for (int x = 0; x < VEC; ++x) acc[x] += red[q * lanes + lane][x];
      }
    }
    if (part == 0 && active) {
#pragma unroll
      for (int x = 0; x < VEC; ++x) {
        if (ADAM) {
          const float m = fmaf(ada.beta1, St[o + x], (1.f - ada.beta1) * acc[x]);
          const float v = fmaf(ada.beta2, Vt[o + x], (1.f - ada.beta2) * acc[x] * acc[x]);
          St[o + x] = m;
          Vt[o + x] = v;
          G[o + x] = g_old[x] - lr * (m * ada.corr1) / (sqrtf(v * ada.corr2) + ada.eps);
        } else if (ADA) {
          const float sq = fmaf(acc[x], acc[x], St[o + x]);
          St[o + x] = sq;
          G[o + x] = g_old[x] - lr * acc[x] / (sqrtf(sq) + ada.eps);
        } else {
          G[o + x] = fmaf(-lr, acc[x], g_old[x]);
        }
      }
    }
    if (parts > 1) __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// host-side launchers

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline int grid_for(int64_t work_items, int cap) {
  return (int)std::max<int64_t>(1, std::min<int64_t>(work_items, cap));
}
constexpr int kGridCap = 256 * 8;  // persistent blocks: 8 per compute unit
constexpr size_t kLdsBudget = 64 * 1024;  // dynamic LDS a block of the staged kernels may ask for

void launch_prefix_fwd(const Plan& pl, const Workspace& ws, const float* g1, const float* g2, int B,
                       hipStream_t st) {
  const int grid = grid_for(cdiv(std::min<int64_t>(B, pl.maxQ), kChunk2) + pl.sh.n2, kGridCap);
  k_prefix_fwd<<<grid, kThreads, 0, st>>>(pl.sh, g1, g2, ws.c2_desc, ws.c2_item, ws.P, ws.ctr);
}

void launch_row_fwd(const Plan& pl, const Workspace& ws, const float* g3, int B, float* out,
                    hipStream_t st) {
  const int tiles = cdiv(B, kTileSlots);
  const int grid = grid_for(cdiv(tiles, kWavesPerBlock), kGridCap);
  const Shape& s = pl.sh;
  const size_t per_wave = ((size_t)s.D + (size_t)s.M * (s.r2 + 1) + s.S3) * sizeof(float);
  if (per_wave <= kLdsBudget) {
    const int wpb = (int)std::min<size_t>(kWavesPerBlock, kLdsBudget / per_wave);
    const size_t staged = wpb * per_wave;
    // one wavefront per distinct id (at most B of them) and per tile of slots
    const int jobs = B + cdiv(B, kTileSlots) + 1;
    k_row_fwd_staged<<<grid_for(cdiv(jobs, wpb), kGridCap * 4), wpb * kWave, staged, st>>>(
        s, B, g3, ws.P, ws.s_u, ws.val[(pl.passes - 1) & 1], ws.u_rs, ws.u_i3, ws.u_q, out, ws.ctr);
    return;
  }
  const size_t lds = (size_t)kWavesPerBlock * pl.sh.D * sizeof(float);
  k_row_fwd<<<grid, kThreads, lds, st>>>(pl.sh, B, g3, ws.P, ws.s_u, ws.val[(pl.passes - 1) & 1],
                                         ws.u_i3, ws.u_q, out, ws.ctr);
}

void launch_gsum(const Plan& pl, const Workspace& ws, const float* grad, int B, hipStream_t st) {
  const int tiles = cdiv(B, kTileSlots);
  const int grid = grid_for(cdiv(tiles, kWavesPerBlock), kGridCap);
  const uint32_t* perm = ws.val[(pl.passes - 1) & 1];
  const size_t lds = (size_t)kWavesPerBlock * pl.sh.D * sizeof(float);
  k_gsum<<<grid, kThreads, lds, st>>>(pl.sh, B, grad, ws.s_u, perm, ws.u_rs, ws.gsum, ws.carry,
                                      ws.ctr);
}

void launch_gsum_fix(const Plan& pl, const Workspace& ws, int B, hipStream_t st) {
  const int grid = grid_for(cdiv(B, kTileSlots), kGridCap);
  k_gsum_fix<<<grid, kThreads, 0, st>>>(pl.sh, ws.s_u, ws.u_rs, ws.carry, ws.gsum, ws.ctr);
}

void launch_u_bwd(const Plan& pl, const Workspace& ws, const float* g3, const float* grad, int B,
                  hipStream_t st) {
  const int grid = grid_for(cdiv(std::min<int64_t>(B, pl.maxQ), kWavesPerBlock), kGridCap * 4);
  k_u_bwd<<<grid, kThreads, 0, st>>>(pl.sh, g3, grad, ws.gsum, ws.u_code, ws.u_i3, ws.q_us, ws.dPsum,
                                     ws.ctr);
}

void launch_dg3(const Plan& pl, const Workspace& ws, const float* grad, int B, hipStream_t st) {
  const int grid = grid_for(cdiv(B, chunk3_fill(B)) + pl.sh.n3, kGridCap);
  const size_t per = ((size_t)pl.sh.PN + pl.sh.D) * sizeof(float);
  if (per <= kLdsBudget) {
    const int group = (int)std::min<size_t>(4, kLdsBudget / per);
    k_dg3_staged<<<grid, kThreads, group * per, st>>>(pl.sh, group, ws.P, grad, ws.gsum, ws.c3_item,
                                                      ws.c3_desc, ws.part3, ws.ctr);
    return;
  }
  k_dg3<<<grid, kThreads, 0, st>>>(pl.sh, ws.P, grad, ws.gsum, ws.c3_item, ws.c3_desc, ws.part3,
                                   ws.ctr);
}

void launch_prefix_bwd(const Plan& pl, const Workspace& ws, const float* g1, const float* g2, int B,
                       hipStream_t st) {
  const int grid = grid_for(cdiv(std::min<int64_t>(B, pl.maxQ), kChunk2) + pl.sh.n2, kGridCap);
  k_prefix_bwd<<<grid, kThreads, 0, st>>>(pl.sh, g1, g2, ws.dPsum, ws.c2_desc, ws.c2_item,
                                          ws.dg1part, ws.part2, ws.ctr);
}

void launch_sgd(const Plan& pl, const Workspace& ws, float* g1, float* g2, float* g3, float lr,
                const UpdateRule& ada, hipEvent_t stop, hipStream_t st) {
  const Shape& s = pl.sh;
  const bool vec = (s.S1 % 4 == 0) && (s.S2 % 4 == 0) && (s.S3 % 4 == 0);
  const int span = kThreads * (vec ? 4 : 1);
  const int64_t jobs = (int64_t)s.n3 * cdiv(s.S3, span) + (int64_t)s.n2 * cdiv(s.S2, span) +
                       (int64_t)s.n1 * cdiv(s.S1, span);
  const int grid = grid_for(jobs, 1 << 16);
  // with `stop` the kernel's own completion signal serves as that event: no separate event packet
  // has to pass through the stream behind the kernel
#define TT_SGD(V, A)                                                                               \
  do {                                                                                             \
    if (stop != nullptr)                                                                           \
      hipExtLaunchKernelGGL((k_sgd<V, A>), dim3(grid), dim3(kThreads), 0, st, nullptr, stop, 0,    \
                            pl.sh, lr, ada, g1, g2, g3, (const float*)ws.part3,                   \
                            (const int*)ws.c3_start, (const float*)ws.part2,                      \
                            (const int*)ws.c2_start, (const float*)ws.dg1part,                    \
                            (const int*)ws.g1_first, (const int*)ws.g1_end, ws.ctr);              \
    else                                                                                           \
      k_sgd<V, A><<<grid, kThreads, 0, st>>>(pl.sh, lr, ada, g1, g2, g3, ws.part3, ws.c3_start,    \
                                             ws.part2, ws.c2_start, ws.dg1part, ws.g1_first,       \
                                             ws.g1_end, ws.ctr);                                   \
  } while (0)
  if (ada.kind == kUpdateAdam) {
    if (vec) TT_SGD(4, kUpdateAdam); else TT_SGD(1, kUpdateAdam);
  } else if (ada.kind == kUpdateAdagrad) {
    if (vec) TT_SGD(4, kUpdateAdagrad); else TT_SGD(1, kUpdateAdagrad);
  } else {
    if (vec) TT_SGD(4, kUpdateSgd); else TT_SGD(1, kUpdateSgd);
  }
#undef TT_SGD
}

}  // namespace ttemb

// Arithmetic kernels of the TT-embedding path for any table shape (gfx950, fp32 on the vector ALUs).
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

// ---------------------------------------------------------------------------------------------
// forward

// P_q = A * Bm, A = G1[i1] (d1 x r1), Bm = G2[i2] (r1 x d2*r2).  Prefixes are visited in by-i2
// order so that neighbouring blocks read the same G2 slice.
__global__ __launch_bounds__(kThreads) void k_prefix_fwd(Shape sh, const float* __restrict__ g1,
                                                         const float* __restrict__ g2,
                                                         const int* __restrict__ g2_list,
                                                         const int* __restrict__ q_i1,
                                                         const int* __restrict__ q_i2,
                                                         float* __restrict__ P,
                                                         const Counters* __restrict__ ctr) {
  const int Q = ctr->Q;
  for (int k = blockIdx.x; k < Q; k += gridDim.x) {
    const int q = g2_list[k];
    const float* A = g1 + (size_t)q_i1[q] * sh.S1;
    const float* Bm = g2 + (size_t)q_i2[q] * sh.S2;
    float* Pq = P + (size_t)q * sh.PN;
    for (int o = threadIdx.x; o < sh.PN; o += kThreads) {
      const int j1 = o / sh.W, col = o % sh.W;
      float acc = 0.f;
      for (int a = 0; a < sh.r1; ++a) acc = fmaf(A[j1 * sh.r1 + a], Bm[a * sh.W + col], acc);
      Pq[o] = acc;
    }
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

// dPsum_q = sum over the unique ids u of prefix q of g_u * G3[i3(u)]^T, g_u read as (d1*d2) x d3.
__global__ __launch_bounds__(kThreads) void k_u_bwd(Shape sh, const float* __restrict__ g3,
                                                    const float* __restrict__ grad,
                                                    const float* __restrict__ gsum,
                                                    const int* __restrict__ u_code,
                                                    const int* __restrict__ u_i3,
                                                    const int* __restrict__ q_us,
                                                    float* __restrict__ dPsum,
                                                    const Counters* __restrict__ ctr) {
  const int Q = ctr->Q;
  for (int q = blockIdx.x; q < Q; q += gridDim.x) {
    const int u0 = q_us[q], u1 = q_us[q + 1];
    for (int o = threadIdx.x; o < sh.PN; o += kThreads) {
      const int m = o / sh.r2, c = o % sh.r2;
      float acc = 0.f;
      for (int u = u0; u < u1; ++u) {
        const float* g = grad_of_unique(u, u_code, grad, gsum, sh.D) + m * sh.d3;
        const float* C = g3 + (size_t)u_i3[u] * sh.S3 + c * sh.d3;
        for (int j3 = 0; j3 < sh.d3; ++j3) acc = fmaf(g[j3], C[j3], acc);
      }
      dPsum[(size_t)q * sh.PN + o] = acc;
    }
  }
}

// part3[c] = sum over the unique ids u of chunk c (all with one i3) of P_q(u)^T g_u   (r2 x d3)
__global__ __launch_bounds__(kThreads) void k_dg3(Shape sh, const float* __restrict__ P,
                                                  const float* __restrict__ grad,
                                                  const float* __restrict__ gsum,
                                                  const int* __restrict__ u_code,
                                                  const int* __restrict__ u_q,
                                                  const int* __restrict__ g3_list,
                                                  const int4* __restrict__ c3_desc,
                                                  float* __restrict__ part3,
                                                  const Counters* __restrict__ ctr) {
  const int nchunk = ctr->nchunk3;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int4 desc = c3_desc[c];
    const int k0 = desc.y, k1 = desc.y + desc.z;
    for (int o = threadIdx.x; o < sh.S3; o += kThreads) {
      const int cc = o / sh.d3, j3 = o % sh.d3;
      float acc = 0.f;
      for (int k = k0; k < k1; ++k) {
        const int u = g3_list[k];
        const float* Pq = P + (size_t)u_q[u] * sh.PN + cc;
        const float* g = grad_of_unique(u, u_code, grad, gsum, sh.D) + j3;
        for (int m = 0; m < sh.M; ++m) acc = fmaf(Pq[m * sh.r2], g[m * sh.d3], acc);
      }
      part3[(size_t)c * sh.S3 + o] = acc;
    }
  }
}

// For the prefixes q of chunk c (all with one i2, Bm = G2[i2]):
//   dg1part[q] = dPsum_q * Bm^T                      (d1 x r1), one per prefix
//   part2[c]   = sum over q of G1[i1(q)]^T * dPsum_q  (r1 x d2*r2)
__global__ __launch_bounds__(kThreads) void k_prefix_bwd(Shape sh, const float* __restrict__ g1,
                                                         const float* __restrict__ g2,
                                                         const float* __restrict__ dPsum,
                                                         const int* __restrict__ q_i1,
                                                         const int* __restrict__ g2_list,
                                                         const int4* __restrict__ c2_desc,
                                                         float* __restrict__ dg1part,
                                                         float* __restrict__ part2,
                                                         const Counters* __restrict__ ctr) {
  const int nchunk = ctr->nchunk2;
  for (int c = blockIdx.x; c < nchunk; c += gridDim.x) {
    const int4 desc = c2_desc[c];
    const int bin = desc.x, k0 = desc.y, k1 = desc.y + desc.z;
    const float* Bm = g2 + (size_t)bin * sh.S2;
    for (int k = k0; k < k1; ++k) {
      const int q = g2_list[k];
      const float* dP = dPsum + (size_t)q * sh.PN;
      for (int o = threadIdx.x; o < sh.S1; o += kThreads) {
        const int j1 = o / sh.r1, a = o % sh.r1;
        float acc = 0.f;
        for (int col = 0; col < sh.W; ++col)
          acc = fmaf(dP[j1 * sh.W + col], Bm[a * sh.W + col], acc);
        dg1part[(size_t)q * sh.S1 + o] = acc;
      }
    }
    for (int o = threadIdx.x; o < sh.S2; o += kThreads) {
      const int a = o / sh.W, col = o % sh.W;
      float acc = 0.f;
      for (int k = k0; k < k1; ++k) {
        const int q = g2_list[k];
        const float* A = g1 + (size_t)q_i1[q] * sh.S1 + a;
        const float* dP = dPsum + (size_t)q * sh.PN + col;
        for (int j1 = 0; j1 < sh.d1; ++j1) acc = fmaf(A[j1 * sh.r1], dP[j1 * sh.W], acc);
      }
      part2[(size_t)c * sh.S2 + o] = acc;
    }
  }
}

// Adds up the partial gradients of every touched slice and applies the update: the SGD step, or
// with ADA the Adagrad step  S += dG^2,  G -= lr * dG / (sqrt(S) + eps)  on the same entries.
// A job owns up to 256*VEC consecutive entries of one slice (VEC = 4 when slice sizes allow 16-byte
// accesses, else 1).  Its threads are arranged as `parts` groups side by side on the entries; the
// job's list of partials (chunks for G3 and G2, prefixes for G1) is dealt round-robin to the
// groups, whose sums are then added in group order.  parts depends on the slice size only and
// every group walks its share in list order, so the order of each sum is fixed by the list length.
// Jobs: n3*cdiv(S3, span) for G3, then n2*cdiv(S2, span) for G2, then n1*cdiv(S1, span) for G1.
template <int VEC, bool ADA>
__global__ __launch_bounds__(kThreads) void k_sgd(Shape sh, float lr, Adagrad ada,
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
    float* St = nullptr;  // Adagrad state of the slice
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
        if (ADA) {
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

void launch_prefix_fwd(const Plan& pl, const Workspace& ws, const float* g1, const float* g2, int B,
                       hipStream_t st) {
  const int grid = grid_for(std::min<int64_t>(B, pl.maxQ), kGridCap);
  k_prefix_fwd<<<grid, kThreads, 0, st>>>(pl.sh, g1, g2, ws.g2_list, ws.q_i1, ws.q_i2, ws.P, ws.ctr);
}

void launch_row_fwd(const Plan& pl, const Workspace& ws, const float* g3, int B, float* out,
                    hipStream_t st) {
  const int tiles = cdiv(B, kTileSlots);
  const int grid = grid_for(cdiv(tiles, kWavesPerBlock), kGridCap);
  const size_t lds = (size_t)kWavesPerBlock * pl.sh.D * sizeof(float);
  k_row_fwd<<<grid, kThreads, lds, st>>>(pl.sh, B, g3, ws.P, ws.s_u, ws.val[(pl.passes - 1) & 1],
                                         ws.u_i3, ws.u_q, out, ws.ctr);
}

void launch_gsum(const Plan& pl, const Workspace& ws, const float* grad, int B, hipStream_t st) {
  const int tiles = cdiv(B, kTileSlots);
  const int grid = grid_for(cdiv(tiles, kWavesPerBlock), kGridCap);
  const size_t lds = (size_t)kWavesPerBlock * pl.sh.D * sizeof(float);
  k_gsum<<<grid, kThreads, lds, st>>>(pl.sh, B, grad, ws.s_u, ws.val[(pl.passes - 1) & 1], ws.u_rs,
                                      ws.gsum, ws.carry, ws.ctr);
}

void launch_gsum_fix(const Plan& pl, const Workspace& ws, int B, hipStream_t st) {
  const int grid = grid_for(cdiv(B, kTileSlots), kGridCap);
  k_gsum_fix<<<grid, kThreads, 0, st>>>(pl.sh, ws.s_u, ws.u_rs, ws.carry, ws.gsum, ws.ctr);
}

void launch_u_bwd(const Plan& pl, const Workspace& ws, const float* g3, const float* grad, int B,
                  hipStream_t st) {
  const int grid = grid_for(std::min<int64_t>(B, pl.maxQ), kGridCap);
  k_u_bwd<<<grid, kThreads, 0, st>>>(pl.sh, g3, grad, ws.gsum, ws.u_code, ws.u_i3, ws.q_us, ws.dPsum,
                                     ws.ctr);
}

void launch_dg3(const Plan& pl, const Workspace& ws, const float* grad, int B, hipStream_t st) {
  const int grid = grid_for(cdiv(B, kChunk3) + pl.sh.n3, kGridCap);
  k_dg3<<<grid, kThreads, 0, st>>>(pl.sh, ws.P, grad, ws.gsum, ws.u_code, ws.u_q, ws.g3_list,
                                   ws.c3_desc, ws.part3, ws.ctr);
}

void launch_prefix_bwd(const Plan& pl, const Workspace& ws, const float* g1, const float* g2, int B,
                       hipStream_t st) {
  const int grid = grid_for(cdiv(std::min<int64_t>(B, pl.maxQ), kChunk2) + pl.sh.n2, kGridCap);
  k_prefix_bwd<<<grid, kThreads, 0, st>>>(pl.sh, g1, g2, ws.dPsum, ws.q_i1, ws.g2_list, ws.c2_desc,
                                          ws.dg1part, ws.part2, ws.ctr);
}

void launch_sgd(const Plan& pl, const Workspace& ws, float* g1, float* g2, float* g3, float lr,
                const Adagrad& ada, hipEvent_t stop, hipStream_t st) {
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
  if (ada.s1 != nullptr) {
    if (vec) TT_SGD(4, true); else TT_SGD(1, true);
  } else {
    if (vec) TT_SGD(4, false); else TT_SGD(1, false);
  }
#undef TT_SGD
}

}  // namespace ttemb

// Device calibration for benchmarks: what a plain streaming copy and a register-resident fp32
// matrix-core loop reach on the device the handle lives on.  Roofline fractions can then be quoted
// against measured peaks beside the nominal ones.  Not on the lookup path.
#include <algorithm>

#include "tt_emb_internal.h"

namespace ttemb {

typedef float f4c __attribute__((ext_vector_type(4)));
typedef float f16c __attribute__((ext_vector_type(16)));

// dst[i] = src[i] over n 16-byte words, grid-stride, four loads in flight per thread
__global__ __launch_bounds__(256) void k_calib_copy(const f4c* __restrict__ src, f4c* __restrict__ dst,
                                                   size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {
    const f4c a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

// iters rounds of four independent v_mfma_f32_32x32x2f32 chains per wavefront (operands in
// registers, no memory traffic); one float per thread is stored so that nothing is optimised away
__global__ __launch_bounds__(256) void k_calib_mfma(float* __restrict__ sink, int iters) {
  const float a = 1.0f + (float)(threadIdx.x % 7) * 0.125f, b = 0.5f + (float)(threadIdx.x % 5) * 0.25f;
  f16c acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[k][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[k], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[k][v];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Gathers of 1 KiB records (one 16-byte word per lane, a whole record per load instruction) at
// pseudo-random places of a table, eight records in flight per wavefront, nothing reused in the
// vector L1 - the access pattern of the per-id operand gathers of the row and gradient kernels.
// With a table that stays in every XCD's L2 this measures the path L2 -> L1; with a table beyond
// the L2s, what the fabric behind them (Infinity Cache, HBM) delivers to such gathers.
__global__ __launch_bounds__(256) void k_calib_gather(const f4c* __restrict__ table, unsigned rec_mask,
                                                     int iters, float* __restrict__ sink) {
  const unsigned lane = threadIdx.x % 64;
  unsigned state = (blockIdx.x * 4u + threadIdx.x / 64u) * 2654435761u + 12345u;  // per wavefront
  f4c acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    f4c v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      state = state * 1664525u + 1013904223u;
      const unsigned rec = (state >> 8) & rec_mask;
      v[k] = table[(size_t)rec * 64 + lane];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += v[k];
  }
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

// Best of `reps` timed launches each; returns a HIP error or hipSuccess.
hipError_t calibrate(void* buf, size_t bytes, hipStream_t st, double* copy_bytes_per_s,
                     double* mfma_flops_per_s, double* gather_bytes_per_s,
                     double* far_gather_bytes_per_s) {
  hipEvent_t a = nullptr, b = nullptr;
  hipError_t e = hipEventCreate(&a);
  if (e == hipSuccess) e = hipEventCreate(&b);
  const int reps = 5;
  double best_copy = 0.0, best_mfma = 0.0;
  // copy: first half of the buffer to the second half
  const size_t words = bytes / 32;  // 16-byte words per half
  const int grid = 256 * 16;
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(a, st);
    if (e != hipSuccess) break;
    k_calib_copy<<<grid, 256, 0, st>>>((const f4c*)buf, (f4c*)buf + words, words);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(b, st);
    if (e == hipSuccess) e = hipEventSynchronize(b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
    if (e == hipSuccess && ms > 0.f)
      best_copy = std::max(best_copy, 2.0 * (double)words * 16.0 / (ms * 1e-3));  // read + write
  }
  // matrix cores: 256 CUs x 8 blocks x 4 wavefronts, 4 chains x iters MFMAs of 32*32*2*2 flops
  const int mgrid = 256 * 8, iters = 4096;
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(a, st);
    if (e != hipSuccess) break;
    k_calib_mfma<<<mgrid, 256, 0, st>>>((float*)buf, iters);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(b, st);
    if (e == hipSuccess) e = hipEventSynchronize(b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
    const double flops = (double)mgrid * 4 /*wavefronts*/ * 4 /*chains*/ * iters * (32.0 * 32 * 2 * 2);
    if (e == hipSuccess && ms > 0.f) best_mfma = std::max(best_mfma, flops / (ms * 1e-3));
  }
  // gathers: a 1 MiB table (1024 records: resident in every L2), then a 64 MiB table (65,536
  // records: beyond the L2s, inside the Infinity Cache) at the start of the buffer; the results go
  // to the buffer's last 2 MiB
  double best_gather[2] = {0.0, 0.0};
  const int ggrid = 256 * 8, giters = 256;
  float* sink = (float*)((char*)buf + bytes - ((size_t)2 << 20));
  for (int t = 0; t < 2 && e == hipSuccess; ++t) {
    const unsigned mask = t == 0 ? 1023u : 65535u;
    if (t == 1 && bytes < ((size_t)66 << 20)) break;  // buffer too small for the large table
    for (int r = 0; r < reps && e == hipSuccess; ++r) {
      e = hipEventRecord(a, st);
      if (e != hipSuccess) break;
      k_calib_gather<<<ggrid, 256, 0, st>>>((const f4c*)buf, mask, giters, sink);
      e = hipGetLastError();
      if (e == hipSuccess) e = hipEventRecord(b, st);
      if (e == hipSuccess) e = hipEventSynchronize(b);
      float ms = 0.f;
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
      const double gbytes = (double)ggrid * 4 /*wavefronts*/ * giters * 8 * 1024.0;
      if (e == hipSuccess && ms > 0.f) best_gather[t] = std::max(best_gather[t], gbytes / (ms * 1e-3));
    }
  }
  if (a) (void)hipEventDestroy(a);
  if (b) (void)hipEventDestroy(b);
  *gather_bytes_per_s = best_gather[0];
  *far_gather_bytes_per_s = best_gather[1];
  *copy_bytes_per_s = best_copy;
  *mfma_flops_per_s = best_mfma;
  return e;
}

}  // namespace ttemb

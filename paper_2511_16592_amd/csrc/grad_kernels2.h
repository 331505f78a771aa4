// Helpers of the gradient pass.
//
//   split_chunks_per_part   how the live transitions are split over the workgroups of a weight-gradient contraction
//   reduce_jobs_kernel, reduce_dw1_ising_kernel   fixed-order sums of the split partial tiles
// The weight-gradient contractions and the input-gradient products are in grad_kernels4.h (bf16 matrix cores,
// three-piece arithmetic).
#pragma once
#include "gfnx_device.h"
#include "grad_kernels.h"

namespace gfnx {

// The live transitions are cut into chunks of 32 rows and the chunks into at most S parts of at least 3
// chunks each, so that short batches do not pay for S partial tiles.
__device__ __forceinline__ int split_chunks_per_part(int chunks, int S) {
  const int per = (chunks + S - 1) / S;
  return per < 3 ? 3 : per;
}

// out[p*Q + q] = sum_s part[s][p][q], q < Q.  A block of 256 threads finishes 64 groups of four outputs: thread
// (o, sg) sums the parts sg, sg+4, sg+8, ... of group o (four loads in flight), and the four sub-sums meet in LDS in
// a fixed order, so the result does not depend on the launch.  grid = ceil(P * QTOT / 4 / 64) blocks.
__device__ __forceinline__ void reduce2_block(const float* __restrict__ part, int S, int P, int QTOT, int Q,
                                              float* __restrict__ out, const int* __restrict__ hdr, int block,
                                              f32x4 (*red)[64]) {
  if (hdr) {  // partials come from a split over the live transitions: only the parts that hold some were written
    const int chunks = (hdr[kHdrNLive] + 31) / 32;
    const int per = split_chunks_per_part(chunks, S);
    S = (chunks + per - 1) / per;
  }
  const int qv = QTOT >> 2;
  const size_t total = (size_t)P * qv;
  const size_t stride = (size_t)P * QTOT;
  const int o = threadIdx.x & 63, sg = threadIdx.x >> 6;
  const size_t i = (size_t)block * 64 + o;
  const bool live = i < total;
  const int p = live ? (int)(i / qv) : 0, q4 = live ? (int)(i % qv) * 4 : 0;
  f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
  if (live && q4 < Q) {
    const float* src = part + (size_t)p * QTOT + q4;
    int s = sg;
    for (; s + 12 < S; s += 16) {
      a0 += *(const f32x4*)&src[(size_t)s * stride];
      a1 += *(const f32x4*)&src[(size_t)(s + 4) * stride];
      a2 += *(const f32x4*)&src[(size_t)(s + 8) * stride];
      a3 += *(const f32x4*)&src[(size_t)(s + 12) * stride];
    }
    for (; s < S; s += 4) a0 += *(const f32x4*)&src[(size_t)s * stride];
  }
  const f32x4 v = (a0 + a1) + (a2 + a3);
  if (sg > 0) red[sg - 1][o] = v;
  __syncthreads();
  if (sg == 0 && live && q4 < Q) {
    const f32x4 t = (v + red[0][o]) + (red[1][o] + red[2][o]);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (q4 + k < Q) out[(size_t)p * Q + q4 + k] = t[k];
  }
}

// Several such reductions in one launch (the weight and bias gradients of all layers at the end of the pass):
// job j owns the blocks [first[j], first[j+1]).
constexpr int kMaxReduceJobs = 6;
struct ReduceJobs {
  const float* part[kMaxReduceJobs];
  float* out[kMaxReduceJobs];
  int S[kMaxReduceJobs], P[kMaxReduceJobs], QTOT[kMaxReduceJobs], Q[kMaxReduceJobs];
  int first[kMaxReduceJobs + 1];
  int n;
};
__global__ __launch_bounds__(256) void reduce_jobs_kernel(const ReduceJobs jobs, const int* __restrict__ hdr) {
  __shared__ f32x4 red[3][64];
  int j = 0;
  while (j + 1 < jobs.n && (int)blockIdx.x >= jobs.first[j + 1]) ++j;
  reduce2_block(jobs.part[j], jobs.S[j], jobs.P[j], jobs.QTOT[j], jobs.Q[j], jobs.out[j], hdr,
                (int)blockIdx.x - jobs.first[j], red);
}

// Ising dW1 from the partial tiles of the one-hot contraction (fixed order over the parts that were written):
// tile rows 2*site, 2*site+1 are the spin rows 3*site, 3*site+2 of dW1; the unassigned row 3*site+1 is db1 minus
// the two (db1 = column sums of G1, reduced before this kernel runs).  Four columns per thread.
__global__ __launch_bounds__(256) void reduce_dw1_ising_kernel(const float* __restrict__ part, int S, int P, int QTOT,
                                                               int H1, const int* __restrict__ hdr,
                                                               const float* __restrict__ db1, float* __restrict__ dW1) {
  __shared__ f32x4 red[3][2][64];
  const int chunks = (hdr[kHdrNLive] + 31) / 32;
  const int per = split_chunks_per_part(chunks, S);
  S = (chunks + per - 1) / per;
  const size_t stride = (size_t)P * QTOT;
  const int qv = H1 >> 2;
  const size_t total = (size_t)(P / 2) * qv;
  const int o = threadIdx.x & 63, sg = threadIdx.x >> 6;  // as in reduce2_block: 64 outputs x 4 groups of parts
  const size_t i = (size_t)blockIdx.x * 64 + o;
  const bool live = i < total;
  const int u = live ? (int)(i / qv) : 0, q = live ? (int)(i % qv) * 4 : 0;
  f32x4 m0 = {0.f, 0.f, 0.f, 0.f}, m1 = m0, p0 = m0, p1 = m0;
  if (live) {
    const float* src = part + (size_t)(2 * u) * QTOT + q;
    int s = sg;
    for (; s + 4 < S; s += 8) {
      m0 += *(const f32x4*)&src[(size_t)s * stride];
      p0 += *(const f32x4*)&src[(size_t)s * stride + QTOT];
      m1 += *(const f32x4*)&src[(size_t)(s + 4) * stride];
      p1 += *(const f32x4*)&src[(size_t)(s + 4) * stride + QTOT];
    }
    for (; s < S; s += 4) {
      m0 += *(const f32x4*)&src[(size_t)s * stride];
      p0 += *(const f32x4*)&src[(size_t)s * stride + QTOT];
    }
  }
  f32x4 mi = m0 + m1, pl = p0 + p1;
  if (sg > 0) { red[sg - 1][0][o] = mi; red[sg - 1][1][o] = pl; }
  __syncthreads();
  if (sg == 0 && live) {
    mi = (mi + red[0][0][o]) + (red[1][0][o] + red[2][0][o]);
    pl = (pl + red[0][1][o]) + (red[1][1][o] + red[2][1][o]);
    *(f32x4*)&dW1[(size_t)(3 * u) * H1 + q] = mi;
    *(f32x4*)&dW1[(size_t)(3 * u + 2) * H1 + q] = pl;
    *(f32x4*)&dW1[(size_t)(3 * u + 1) * H1 + q] = *(const f32x4*)&db1[q] - mi - pl;
  }
}

}  // namespace gfnx

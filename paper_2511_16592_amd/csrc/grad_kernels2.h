// Helpers and binary32 matrix-core kernels of the gradient pass.
//
//   split_chunks_per_part   how the live transitions are split over the workgroups of a weight-gradient contraction
//   reduce_jobs_kernel, reduce_dw1_ising_kernel   fixed-order sums of the split partial tiles
//   gemm_nt2k_kernel        Out = (G W^T) . [act > 0] for contraction lengths above 256 (512-wide networks)
// The weight-gradient contractions and the input-gradient products up to 256 are in grad_kernels4.h (bf16 matrix
// cores, three-piece arithmetic).
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

// Input-gradient product for contraction lengths above 256 (K <= 512), binary32 matrix instructions:
// for each live row i, Out[i][p] = (sum_q Gin[i][q] * W[p][q]) * [act[i][p] > 0], written over the stored activation,
// in tiles of 32 rows x 128 columns; W is given transposed (Wt[q][p], P columns per row) so that the register slices
// load coalesced; the ReLU derivative comes from the 1-bit sign masks the rollout recorded (word k of a row holds bit
// l for unit 4l+k), so the epilogue only stores.  The eight waves are 4 column blocks x 2 halves of the contraction: wave (cb, kh) keeps
// W[32 columns of cb][q in 256 kh .. 256 kh + 255] in 128 registers; the two half-sums of a column block meet in
// LDS and the kh = 0 wave stores.  grid = (row-tile workers (grid-stride), ceil(P / 128)).
__global__ __launch_bounds__(512) void gemm_nt2k_kernel(const float* __restrict__ Gin, int ldgi, int K,
                                                        const float* __restrict__ Wt, int Kvalid,
                                                        float* __restrict__ ActOut, int ldo, int P,
                                                        const unsigned long long* __restrict__ mask, int MW,
                                                        const int* __restrict__ rows, const int* __restrict__ hdr) {
  constexpr int KP = 514, R = 32;  // LDS row pitch in floats (even, 2 mod 32), rows per tile
  extern __shared__ float smem[];
  float* GS = smem;                          // [R][KP]
  f32x16* XCH = (f32x16*)(smem + R * KP);    // [4 column blocks][64 lanes]: half-sums of the kh = 1 waves
  int* ridb = (int*)(XCH + 4 * 64);          // [3][R] row ids of three consecutive tiles
  uint32_t* MS = (uint32_t*)(ridb + 3 * R);  // [R][4]: the 32-bit halves of the four mask words of this column tile
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cb = w & 3, kh = w >> 2, kk = lane >> 5;
  const int n = hdr[kHdrNLive];
  const int tiles = (n + R - 1) / R;
  const int ct = blockIdx.y;
  const int pl = 32 * cb + (lane & 31);      // column within the tile
  const int pcol = ct * 128 + pl;
  // unit u = 128 ct + pl: mask word 4 (u >> 8) + (u & 3), bit (u & 255) >> 2 = 32 (ct & 1) + (pl >> 2)
  const uint32_t* mask32 = (const uint32_t*)mask + 2 * (4 * (ct >> 1)) + (ct & 1);

  float wreg[128];
#pragma unroll
  for (int s = 0; s < 128; ++s) {
    const int q = 256 * kh + 4 * (s >> 1) + 2 * kk + (s & 1);
    wreg[s] = (q < Kvalid && pcol < P) ? Wt[(size_t)q * P + pcol] : 0.f;
  }

  const int kv = K >> 2;  // f32x4 per row
  f32x4 pre[8];
  uint32_t mpre = 0;
  int idreg = -1;
  auto fetch_ids = [&](int tile) {
    if (tid < R) idreg = (tile < tiles && tile * R + tid < n) ? rows[tile * R + tid] : -1;
  };
  auto load_rows = [&](const int* ids) {
    if (tid < R * 4) {
      const int rr = ids[tid >> 2];
      mpre = rr >= 0 ? mask32[(size_t)rr * MW * 2 + 2 * (tid & 3)] : 0u;
    }
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;  // R rows x 128 quads
      const int rr = ids[i >> 7], c4 = i & 127;
      pre[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (rr >= 0 && c4 < kv) pre[m] = *(const f32x4*)&Gin[(size_t)rr * ldgi + 4 * c4];
    }
  };

  int tile = blockIdx.x;
  fetch_ids(tile);
  if (tid < R) ridb[tid] = idreg;
  lds_barrier();
  load_rows(ridb);
  fetch_ids(tile + gridDim.x);
  for (int it = 0; tile < tiles; tile += gridDim.x, ++it) {
    const int* rid = ridb + R * (it % 3);
    int* rid_next = ridb + R * ((it + 1) % 3);
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;
      float* d = &GS[(i >> 7) * KP + 4 * (i & 127)];
      *(float2*)d = make_float2(pre[m].x, pre[m].y);
      *(float2*)(d + 2) = make_float2(pre[m].z, pre[m].w);
    }
    if (tid < R * 4) MS[tid] = mpre;
    if (tid < R) rid_next[tid] = idreg;
    lds_barrier();
    load_rows(rid_next);
    fetch_ids(tile + 2 * (int)gridDim.x);
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const float* g0 = &GS[(lane & 31) * KP + 256 * kh + 2 * kk];
#pragma unroll
    for (int grp = 0; grp < 16; ++grp) {
      if (256 * kh + 16 * grp < K) {
        float2 a0[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a0[u] = *(const float2*)&g0[16 * grp + 4 * u];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int s2 = 4 * grp + u;
          acc = mfma32(a0[u].x, wreg[2 * s2], acc);
          acc = mfma32(a0[u].y, wreg[2 * s2 + 1], acc);
        }
      }
    }
    if (kh == 1) XCH[cb * 64 + lane] = acc;
    lds_barrier();
    if (kh == 0) {
      const f32x16 other = XCH[cb * 64 + lane];
      if (pcol < P) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 8 * (r >> 2) + 4 * kk + (r & 3);
          const int r0 = rid[i];
          const uint32_t b0 = (MS[i * 4 + (pl & 3)] >> (pl >> 2)) & 1u;
          if (r0 >= 0) ActOut[(size_t)r0 * ldo + pcol] = b0 ? acc[r] + other[r] : 0.f;
        }
      }
    }
    lds_barrier();
  }
}

inline size_t gemm_nt2k_lds_bytes() { return (32 * 514 + 4 * 64 * 16 + 3 * 32 + 32 * 4) * 4; }

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

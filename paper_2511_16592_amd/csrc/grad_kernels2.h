// Matrix-core kernels of the gradient pass (binary32 MFMA, operands staged in LDS).
//
//   gemm_tn2_kernel   dW = X^T G over the live transitions: 8 waves hold a 256 x 256 (or 256 x 32) accumulator
//                     tile in registers (blockIdx.x / .y pick the tile of wider operands), transition rows are
//                     gathered through the row list in chunks of 32 and staged in double-buffered LDS, the rows
//                     two chunks ahead are in flight while the matrix cores work; column sums of G (the bias
//                     gradient) ride along.
//   gemm_nt2_kernel   Out = (G W^T) . [act > 0], contraction length <= 256: each wave keeps a 32-column slice of W
//                     in registers as the MFMA B operand for the whole kernel; tiles of 64 transition rows stream
//                     through LDS.   gemm_nt2k_kernel: the same for contraction lengths up to 512.
//                     (W comes transposed, prepared with the rollout's weights, so that those slices load coalesced)
//   reduce_jobs_kernel, reduce_dw1_ising_kernel   fixed-order sums of the split partial tiles.
// With SCALE the G operand is (2 delta_b / B) * e, formed while the rows are loaded, so the logit-gradient rows
// are never rewritten in HBM.
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

template <int WP, int WQ, int PBW, int QBW, bool SCALE>
__global__ __launch_bounds__(512) void gemm_tn2_kernel(const float* __restrict__ X, int ldx, int P,
                                                       const float* __restrict__ G, int ldg,
                                                       const float* __restrict__ crow,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr,
                                                       int QTOT, float* __restrict__ part,
                                                       float* __restrict__ dbpart) {
  constexpr int PT = WP * PBW * 32, QT = WQ * QBW * 32, KC = 32;
  constexpr int XV = KC * PT / 4 / 512, GV = (KC * QT / 4 + 511) / 512;  // f32x4 per thread per chunk
  static_assert(WP * WQ == 8, "eight waves");
  extern __shared__ float smem[];  // two buffers of [KC][PT] + [KC][QT]
  constexpr int kBuf = KC * (PT + QT);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ptile = blockIdx.x, qtile = blockIdx.y, s = blockIdx.z, S = gridDim.z;
  const int n = hdr[kHdrNLive];
  const int chunks = (n + KC - 1) / KC;
  const int per = split_chunks_per_part(chunks, S);
  const int c0 = s * per, c1 = min(chunks, c0 + per);
  if (c0 >= c1) return;  // parts beyond the live transitions write nothing; the reduction skips them too
  const int pbase = (w / WQ) * PBW * 32, qbase = (w % WQ) * QBW * 32;

  f32x16 acc[PBW][QBW];
#pragma unroll
  for (int a = 0; a < PBW; ++a)
#pragma unroll
    for (int b = 0; b < QBW; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  float dbacc = 0.f;

  // software pipeline: row ids of chunk c+2 and rows of chunk c+1 are in flight while chunk c is multiplied
  f32x4 xr[XV], gr[GV];
  int xid[XV], gid[GV];
  float gcf[GV];  // SCALE: coefficient of the row, from the list that runs parallel to the row list
  auto load_ids = [&](int c) {
#pragma unroll
    for (int m = 0; m < XV; ++m) {
      const int li = c * KC + (tid + 512 * m) / (PT / 4);
      xid[m] = (c < c1 && li < n) ? rows[li] : -1;
    }
#pragma unroll
    for (int m = 0; m < GV; ++m) {
      const int i = tid + 512 * m;
      const int li = c * KC + i / (QT / 4);
      const bool on = c < c1 && i < KC * QT / 4 && li < n;
      gid[m] = on ? rows[li] : -1;
      if (SCALE) gcf[m] = on ? crow[li] : 0.f;
    }
  };
  auto load_rows = [&]() {
#pragma unroll
    for (int m = 0; m < XV; ++m) {
      const int c4 = (tid + 512 * m) % (PT / 4);
      xr[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (xid[m] >= 0 && ptile * PT + 4 * c4 < P) xr[m] = *(const f32x4*)&X[(size_t)xid[m] * ldx + ptile * PT + 4 * c4];
    }
#pragma unroll
    for (int m = 0; m < GV; ++m) {
      const int col = qtile * QT + 4 * ((tid + 512 * m) % (QT / 4));
      gr[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (gid[m] >= 0 && col < ldg) {
        f32x4 v = *(const f32x4*)&G[(size_t)gid[m] * ldg + col];
        if (SCALE) v = v * gcf[m];
        gr[m] = v;
      }
    }
  };
  auto store_chunk = [&](float* XS, float* GS) {
#pragma unroll
    for (int m = 0; m < XV; ++m) {
      const int i = tid + 512 * m;
      *(f32x4*)&XS[(i / (PT / 4)) * PT + 4 * (i % (PT / 4))] = xr[m];
    }
#pragma unroll
    for (int m = 0; m < GV; ++m) {
      const int i = tid + 512 * m;
      if (i < KC * QT / 4) *(f32x4*)&GS[(i / (QT / 4)) * QT + 4 * (i % (QT / 4))] = gr[m];
    }
  };

  // Chunk c is multiplied out of LDS buffer c % 2 while chunk c+1 (already in registers) is written to the other
  // buffer and the rows of chunk c+2 are requested: one barrier per chunk.
  load_ids(c0);
  load_rows();
  load_ids(c0 + 1);
  store_chunk(smem, smem + KC * PT);
  load_rows();          // chunk c0+1
  load_ids(c0 + 2);
  lds_barrier();
  for (int c = c0; c < c1; ++c) {
    const float* XS = smem + ((c - c0) & 1) * kBuf;
    const float* GS = XS + KC * PT;
    float* XSn = smem + ((c - c0 + 1) & 1) * kBuf;
    store_chunk(XSn, XSn + KC * PT);  // chunk c+1 (zeros past the end); its buffer was last read for chunk c-1
    load_rows();                      // chunk c+2, ids already here
    load_ids(c + 3);
#pragma unroll 4
    for (int k = 0; k < KC; k += 2) {
      const int kk = k + (lane >> 5);
      float av[PBW], bv[QBW];
#pragma unroll
      for (int a = 0; a < PBW; ++a) av[a] = XS[kk * PT + pbase + 32 * a + (lane & 31)];
#pragma unroll
      for (int b = 0; b < QBW; ++b) bv[b] = GS[kk * QT + qbase + 32 * b + (lane & 31)];
#pragma unroll
      for (int a = 0; a < PBW; ++a)
#pragma unroll
        for (int b = 0; b < QBW; ++b) acc[a][b] = mfma32(av[a], bv[b], acc[a][b]);
    }
    if (ptile == 0 && tid < QT) {
#pragma unroll 8
      for (int k = 0; k < KC; ++k) dbacc += GS[k * QT + tid];
    }
    lds_barrier();
  }
  float* out = part + (size_t)s * P * QTOT;
#pragma unroll
  for (int a = 0; a < PBW; ++a)
#pragma unroll
    for (int b = 0; b < QBW; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int pi = ptile * PT + pbase + 32 * a + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int qi = qtile * QT + qbase + 32 * b + (lane & 31);
        if (pi < P) out[(size_t)pi * QTOT + qi] = acc[a][b][r];
      }
  if (ptile == 0 && tid < QT) dbpart[(size_t)s * QTOT + qtile * QT + tid] = dbacc;
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

// For each live row i: Out[i][p] = (sum_q Gin[i][q] * W[p][q]) * [act[i][p] > 0], written over the stored
// activation; W is given transposed (Wt[q][p], P columns per row); the ReLU derivative comes from the 1-bit sign masks the rollout recorded (word k of a row holds
// bit l for unit 4l+k), so the epilogue only stores.  Contraction length K <= 256 (rows of Gin hold K floats,
// W rows hold Kvalid <= K).
// grid = (row-tile workers (grid-stride), ceil(P/256)); 8 waves, wave w owns output columns 32w .. 32w+31.
template <bool SCALE>
__global__ __launch_bounds__(512) void gemm_nt2_kernel(const float* __restrict__ Gin, int ldgi, int K,
                                                       const float* __restrict__ Wt, int Kvalid,
                                                       float* __restrict__ ActOut, int ldo, int P,
                                                       const unsigned long long* __restrict__ mask, int MW,
                                                       const float* __restrict__ crow,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr) {
  constexpr int KP = 258;  // LDS row pitch in floats: even (8-byte reads) and 2 mod 32 (conflict-free rows)
  extern __shared__ float smem[];
  float* GSb = smem;                         // [2][64][KP] row tiles, double-buffered
  int* ridb = (int*)(smem + 2 * 64 * KP);    // [4][64] physical row ids of four consecutive tiles
  uint32_t* MSb = (uint32_t*)(ridb + 256);   // [2][64 rows][8]: the four 64-bit mask words of this column tile
  float* cfb = (float*)(MSb + 1024);         // [4][64] coefficients of the same rows (SCALE)
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = hdr[kHdrNLive];
  const int tiles = (n + 63) >> 6;
  const int pcol = blockIdx.y * 256 + 32 * w + (lane & 31);
  const uint32_t* mask32 = (const uint32_t*)mask + (size_t)blockIdx.y * 8;
  const int kk = lane >> 5;

  // B operand: step s consumes contraction index q = 4*(s/2) + 2*kk + (s%2)
  float wreg[128];
#pragma unroll
  for (int s = 0; s < 128; ++s) {
    const int q = 4 * (s >> 1) + 2 * kk + (s & 1);
    wreg[s] = (q < Kvalid && pcol < P) ? Wt[(size_t)q * P + pcol] : 0.f;
  }

  const int kv = K >> 2;               // f32x4 per row
  f32x4 pre[8];
  uint32_t mpre = 0;
  int idreg = -1;
  float cfreg = 0.f;
  auto fetch_ids = [&](int tile) {  // threads 0..63
    if (tid < 64) {
      const bool on = tile < tiles && tile * 64 + tid < n;
      idreg = on ? rows[tile * 64 + tid] : -1;
      if (SCALE) cfreg = on ? crow[tile * 64 + tid] : 0.f;
    }
  };
  auto load_rows = [&](const int* ids, const float* cfs) {
    {
      const int rr = ids[tid >> 3];    // mask tile: 64 rows x 8 words of 32 bits, one per thread
      mpre = rr >= 0 ? mask32[(size_t)rr * MW * 2 + (tid & 7)] : 0u;
    }
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;     // 64 rows x 64 quads
      const int rr = ids[i >> 6], c4 = i & 63;
      pre[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (rr >= 0 && c4 < kv) {
        f32x4 v = *(const f32x4*)&Gin[(size_t)rr * ldgi + 4 * c4];
        if (SCALE) v = v * cfs[i >> 6];
        pre[m] = v;
      }
    }
  };

  // Tile k of this workgroup is row tile blockIdx.x + k * gridDim.x.  In iteration it the matrix cores work on
  // LDS buffer it % 2 while the rows of tile it+1 (in registers since the previous iteration) go to the other
  // buffer, the rows of tile it+2 are requested and the row ids of tile it+4 are fetched: one barrier per tile.
  // Row ids (and coefficients) live in LDS four tiles deep, from the request of a tile's rows to its epilogue.
  const int t0 = blockIdx.x, dt = gridDim.x;
  auto store_tile = [&](int buf) {
    float* GS = GSb + buf * 64 * KP;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;
      float* d = &GS[(i >> 6) * KP + 4 * (i & 63)];
      *(float2*)d = make_float2(pre[m].x, pre[m].y);
      *(float2*)(d + 2) = make_float2(pre[m].z, pre[m].w);
    }
    MSb[buf * 512 + tid] = mpre;
  };
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    fetch_ids(t0 + k * dt);
    if (tid < 64) { ridb[64 * k + tid] = idreg; cfb[64 * k + tid] = cfreg; }
  }
  lds_barrier();
  load_rows(ridb, cfb);
  store_tile(0);
  load_rows(ridb + 64, cfb + 64);
  fetch_ids(t0 + 3 * dt);
  lds_barrier();
  int it = 0;
  for (int tile = t0; tile < tiles; tile += dt, ++it) {
    const int* rid = ridb + 64 * (it & 3);
    const float* GS = GSb + (it & 1) * 64 * KP;
    const uint32_t* MS = MSb + (it & 1) * 512;
    store_tile((it + 1) & 1);
    if (tid < 64) { ridb[64 * ((it + 3) & 3) + tid] = idreg; cfb[64 * ((it + 3) & 3) + tid] = cfreg; }
    load_rows(ridb + 64 * ((it + 2) & 3), cfb + 64 * ((it + 2) & 3));
    fetch_ids(tile + 4 * dt);
    // the 64 rows of the tile as two passes of 32, one accumulator block live at a time
    const int pl = 32 * w + (lane & 31);
    const int mk = pl & 3, ml = pl >> 2;  // unit p = 4l + k of this column tile: bit l of mask word k
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      const float* g0 = &GS[(32 * half + (lane & 31)) * KP + 2 * kk];
      // K is a multiple of 16: one uniform branch per 16 contraction indices, so that inside a group the LDS
      // reads of the later steps are issued under the MFMAs of the earlier ones
#pragma unroll
      for (int grp = 0; grp < 16; ++grp) {
        if (16 * grp < K) {
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
      if (pcol < P) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 32 * half + 8 * (r >> 2) + 4 * kk + (r & 3);
          const int r0 = rid[i];
          const uint32_t b0 = (MS[i * 8 + 2 * mk + (ml >> 5)] >> (ml & 31)) & 1u;
          if (r0 >= 0) ActOut[(size_t)r0 * ldo + pcol] = b0 ? acc[r] : 0.f;
        }
      }
    }
    lds_barrier();
  }
}

// The same product for contraction lengths above 256 (K <= 512): Out = (Gin W^T) . [act > 0] in tiles of 32 rows
// x 128 columns.  The eight waves are 4 column blocks x 2 halves of the contraction: wave (cb, kh) keeps
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

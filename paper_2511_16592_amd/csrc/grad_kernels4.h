// Weight-gradient contraction dW = X^T G on the bf16 matrix cores with binary32-equivalent arithmetic.
//
// Every binary32 operand is cut into three bf16 pieces of 8 significant bits each, x = x_h + x_m + x_l exactly (by
// truncation, as in dw1_onehot_kernel), and a product x * g is formed from the six piece products of weight down to
// 2^-16: x_h g_h, x_h g_m, x_m g_h, x_h g_l, x_l g_h, x_m g_m.  Each piece product is exact (8 x 8 significant bits) and
// is accumulated in binary32 by the matrix core; what is dropped (x_m g_l, x_l g_m, x_l g_l) is below 2^-23 |x g|, the
// size of the rounding error of one binary32 multiply-add.  Per 32 x 32 x 16 block of work, six bf16 instructions
// (6 x 32 = 192 cycles of the matrix pipe) replace eight binary32 ones of 32 x 32 x 2 (8 x 64 = 512 cycles).
//
// One workgroup = 8 waves holds a PT x QT accumulator tile (256 x 256, 256 x 224 or 256 x 32) of
// v_mfma_f32_32x32x16_bf16 blocks in registers (blockIdx.x / .y pick the tile of wider operands); the transitions are
// split over blockIdx.z (split_chunks_per_part), every part writes a partial tile part[s][p][QTOT] and, for
// blockIdx.x = 0, the column sums of G (the bias gradient) dbpart[s][QTOT]; reduce_jobs_kernel sums the parts.  The
// matrix instruction contracts 16 transition rows and wants, per lane, 8 consecutive ROWS of one column: each thread
// therefore loads its column of 8 rows straight from global memory (lanes = consecutive columns: coalesced), splits
// the 8 values once, and writes three 16-byte pieces to LDS in operand order [piece][row octet][column]; every wave
// then reads its operands with 16-byte LDS loads.  Steps of 16 rows are double-buffered in LDS: while the matrix cores
// work on step s, the values of step s+1 (in registers since the previous step) are split and written, and the loads
// of step s+2 are in flight; the row ids run one step further ahead.  One barrier per step.
#pragma once
#include <type_traits>
#include "gfnx_device.h"
#include "grad_kernels.h"
#include "grad_kernels2.h"
#include "grad_kernels3.h"

namespace gfnx {

// x = h + m + l exactly, each with at most 8 significant bits; returned as bf16 bit patterns in the HIGH half of a word
__device__ __forceinline__ void split3(float x, uint32_t& h, uint32_t& m, uint32_t& l) {
  h = __builtin_bit_cast(uint32_t, x) & 0xFFFF0000u;
  const float r1 = x - __builtin_bit_cast(float, h);
  m = __builtin_bit_cast(uint32_t, r1) & 0xFFFF0000u;
  const float r2 = r1 - __builtin_bit_cast(float, m);
  l = __builtin_bit_cast(uint32_t, r2);  // at most 8 significant bits are left: the low half is zero
}

// eight binary32 values (consecutive contraction rows of one column) -> three packed operands of eight bf16
__device__ __forceinline__ void split3x8(const float v[8], u32x4& ph, u32x4& pm, u32x4& pl) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    uint32_t h0, m0, l0, h1, m1, l1;
    split3(v[2 * k], h0, m0, l0);
    split3(v[2 * k + 1], h1, m1, l1);
    ph[k] = (h0 >> 16) | h1;
    pm[k] = (m0 >> 16) | m1;
    pl[k] = (l0 >> 16) | (l1 & 0xFFFF0000u);
  }
}

constexpr int kTn3Step = 16;  // transition rows per matrix instruction / pipeline step

template <int WP, int WQ, int PBW, int QBW>
constexpr size_t gemm_tn3_lds_bytes() {
  return (size_t)2 * 3 * 2 * (WP * PBW * 32 + WQ * QBW * 32) * 16;  // 2 buffers x 3 pieces x 2 row octets x columns
}

template <int WP, int WQ, int PBW, int QBW, bool SCALE>
__global__ __launch_bounds__(512) void gemm_tn3_kernel(const float* __restrict__ X, int ldx, int P,
                                                       const float* __restrict__ G, int ldg,
                                                       const float* __restrict__ crow,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr,
                                                       int QTOT, float* __restrict__ part,
                                                       float* __restrict__ dbpart) {
  constexpr int PT = WP * PBW * 32, QT = WQ * QBW * 32;
  constexpr int XU = (2 * PT + 511) / 512, GU = (2 * QT + 511) / 512;  // (column, row octet) units per thread
  static_assert(WP * WQ == 8, "eight waves");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  constexpr int kBufVecs = 3 * 2 * (PT + QT);  // 16-byte vectors per buffer
  u32x4* lds = (u32x4*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ptile = blockIdx.x, qtile = blockIdx.y, s = blockIdx.z, S = gridDim.z;
  const int n = hdr[kHdrNLive];
  const int chunks = (n + 31) / 32;
  const int per = split_chunks_per_part(chunks, S);
  const int c0 = s * per, c1 = min(chunks, c0 + per);
  if (c0 >= c1) return;  // parts beyond the live transitions write nothing; the reduction skips them too
  const int row0 = 32 * c0, row1 = min(n, 32 * c1);  // this part's slice of the row list
  const int steps = (row1 - row0 + kTn3Step - 1) / kTn3Step;
  const int pbase = (w / WQ) * PBW * 32, qbase = (w % WQ) * QBW * 32;
  const int kg = lane >> 5, l32 = lane & 31;

  f32x16 acc[PBW][QBW];
#pragma unroll
  for (int a = 0; a < PBW; ++a)
#pragma unroll
    for (int b = 0; b < QBW; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  float dbacc[GU];
#pragma unroll
  for (int u = 0; u < GU; ++u) dbacc[u] = 0.f;

  // ---- loader roles: unit u of this thread = (column, row octet) of X and of G
  int xcol[XU], xoct[XU], gcol[GU], goct[GU];
  bool xon[XU], gon[GU];
#pragma unroll
  for (int u = 0; u < XU; ++u) {
    const int i = tid + 512 * u;
    xcol[u] = i % PT; xoct[u] = i / PT;
    xon[u] = i < 2 * PT && ptile * PT + xcol[u] < P;
  }
#pragma unroll
  for (int u = 0; u < GU; ++u) {
    const int i = tid + 512 * u;
    gcol[u] = i % QT; goct[u] = i / QT;
    gon[u] = i < 2 * QT && qtile * QT + gcol[u] < ldg;
  }
  // row ids (and coefficients) of the eight rows of every unit, one step ahead of the values
  int4 xid[XU][2], gid[GU][2];
  f32x4 gcf[GU][2];
  // (loads are unconditional -- a list position past this part's range, or a step past its end, is read at a clamped
  // index and the id replaced by -1; a row id of -1 or a column past the operand is read at row / column 0 and the
  // value replaced by zero -- so that the loop body is branch-free)
  auto load_ids = [&](int step) {
    const int stc = min(step, steps - 1);
    const int lim = step < steps ? row1 : 0;  // list positions >= lim hold no row of this step
#pragma unroll
    for (int u = 0; u < XU; ++u) {
      const int li = row0 + stc * kTn3Step + 8 * min(xoct[u], 1);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int lj = li + 4 * hh;
        int4 v = *(const int4*)&rows[lj];
        v.x = lj < lim ? v.x : -1;
        v.y = lj + 1 < lim ? v.y : -1;
        v.z = lj + 2 < lim ? v.z : -1;
        v.w = lj + 3 < lim ? v.w : -1;
        xid[u][hh] = v;
      }
    }
#pragma unroll
    for (int u = 0; u < GU; ++u) {
      const int li = row0 + stc * kTn3Step + 8 * min(goct[u], 1);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int lj = li + 4 * hh;
        int4 v = *(const int4*)&rows[lj];
        v.x = lj < lim ? v.x : -1;
        v.y = lj + 1 < lim ? v.y : -1;
        v.z = lj + 2 < lim ? v.z : -1;
        v.w = lj + 3 < lim ? v.w : -1;
        gid[u][hh] = v;
        if (SCALE) gcf[u][hh] = *(const f32x4*)&crow[lj];
      }
    }
  };
  // the values are used (masked, scaled, split) one step after their loads are issued; what that needs of the ids
  // and coefficients, which are overwritten in between, is kept beside them
  float xv[XU][8], gv[GU][8], gcv[GU][8];
  uint32_t xok[XU], gok[GU];
  auto load_values = [&]() {
#pragma unroll
    for (int u = 0; u < XU; ++u) {
      const int id[8] = {xid[u][0].x, xid[u][0].y, xid[u][0].z, xid[u][0].w,
                         xid[u][1].x, xid[u][1].y, xid[u][1].z, xid[u][1].w};
      const float* src = X + (xon[u] ? ptile * PT + xcol[u] : 0);
      xok[u] = 0u;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        xv[u][k] = src[(uint64_t)(uint32_t)max(id[k], 0) * (uint32_t)ldx];
        xok[u] |= (uint32_t)(xon[u] && id[k] >= 0) << k;
      }
    }
#pragma unroll
    for (int u = 0; u < GU; ++u) {
      const int id[8] = {gid[u][0].x, gid[u][0].y, gid[u][0].z, gid[u][0].w,
                         gid[u][1].x, gid[u][1].y, gid[u][1].z, gid[u][1].w};
      const float cf[8] = {gcf[u][0].x, gcf[u][0].y, gcf[u][0].z, gcf[u][0].w,
                           gcf[u][1].x, gcf[u][1].y, gcf[u][1].z, gcf[u][1].w};
      const float* src = G + (gon[u] ? qtile * QT + gcol[u] : 0);
      gok[u] = 0u;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        gv[u][k] = src[(uint64_t)(uint32_t)max(id[k], 0) * (uint32_t)ldg];
        gok[u] |= (uint32_t)(gon[u] && id[k] >= 0) << k;
        if (SCALE) gcv[u][k] = cf[k];
      }
    }
  };
  // split the values in hand and write them to LDS buffer `buf` in operand order [piece][row octet][column]
  auto store_step = [&](int buf) {
    u32x4* XS = lds + buf * kBufVecs;
    u32x4* GS = XS + 3 * 2 * PT;
#pragma unroll
    for (int u = 0; u < XU; ++u) {
      if (tid + 512 * u < 2 * PT) {
        u32x4 ph, pm, pl;
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = ((xok[u] >> k) & 1u) ? xv[u][k] : 0.f;
        split3x8(v, ph, pm, pl);
        XS[(0 * 2 + xoct[u]) * PT + xcol[u]] = ph;
        XS[(1 * 2 + xoct[u]) * PT + xcol[u]] = pm;
        XS[(2 * 2 + xoct[u]) * PT + xcol[u]] = pl;
      }
    }
#pragma unroll
    for (int u = 0; u < GU; ++u) {
      if (tid + 512 * u < 2 * QT) {
        u32x4 ph, pm, pl;
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = ((gok[u] >> k) & 1u) ? (SCALE ? gv[u][k] * gcv[u][k] : gv[u][k]) : 0.f;
        split3x8(v, ph, pm, pl);
        GS[(0 * 2 + goct[u]) * QT + gcol[u]] = ph;
        GS[(1 * 2 + goct[u]) * QT + gcol[u]] = pm;
        GS[(2 * 2 + goct[u]) * QT + gcol[u]] = pl;
#pragma unroll
        for (int k = 0; k < 8; ++k) dbacc[u] += v[k];
      }
    }
  };

  // ---- prologue: step 0 in LDS, values of step 1 in flight, ids of step 2 in hand
  load_ids(0);
  load_values();
  load_ids(1);
  store_step(0);
  load_values();
  load_ids(2);
  lds_barrier();
  for (int st = 0; st < steps; ++st) {
    const u32x4* XS = lds + (st & 1) * kBufVecs;
    const u32x4* GS = XS + 3 * 2 * PT;
    store_step((st + 1) & 1);  // step st+1 (zeros past the end); that buffer was last read for step st-1
    load_values();             // step st+2, ids already here
    load_ids(st + 3);
    // the operand pieces of the narrower side of the wave's sub-tile stay in registers, the other side streams
    if constexpr (QBW <= PBW) {
      u32x4 bh[QBW], bm[QBW], bl[QBW];
#pragma unroll
      for (int b = 0; b < QBW; ++b) {
        const int col = qbase + 32 * b + l32;
        bh[b] = GS[(0 * 2 + kg) * QT + col];
        bm[b] = GS[(1 * 2 + kg) * QT + col];
        bl[b] = GS[(2 * 2 + kg) * QT + col];
      }
#pragma unroll
      for (int a = 0; a < PBW; ++a) {
        const int col = pbase + 32 * a + l32;
        const u32x4 ah = XS[(0 * 2 + kg) * PT + col];
        const u32x4 am = XS[(1 * 2 + kg) * PT + col];
        const u32x4 al = XS[(2 * 2 + kg) * PT + col];
#pragma unroll
        for (int b = 0; b < QBW; ++b) {  // smallest products first
          acc[a][b] = mfma32_bf16(am, bm[b], acc[a][b]);
          acc[a][b] = mfma32_bf16(al, bh[b], acc[a][b]);
          acc[a][b] = mfma32_bf16(ah, bl[b], acc[a][b]);
          acc[a][b] = mfma32_bf16(am, bh[b], acc[a][b]);
          acc[a][b] = mfma32_bf16(ah, bm[b], acc[a][b]);
          acc[a][b] = mfma32_bf16(ah, bh[b], acc[a][b]);
        }
      }
    } else {
      u32x4 ah[PBW], am[PBW], al[PBW];
#pragma unroll
      for (int a = 0; a < PBW; ++a) {
        const int col = pbase + 32 * a + l32;
        ah[a] = XS[(0 * 2 + kg) * PT + col];
        am[a] = XS[(1 * 2 + kg) * PT + col];
        al[a] = XS[(2 * 2 + kg) * PT + col];
      }
#pragma unroll
      for (int b = 0; b < QBW; ++b) {
        const int col = qbase + 32 * b + l32;
        const u32x4 bh = GS[(0 * 2 + kg) * QT + col];
        const u32x4 bm = GS[(1 * 2 + kg) * QT + col];
        const u32x4 bl = GS[(2 * 2 + kg) * QT + col];
#pragma unroll
        for (int a = 0; a < PBW; ++a) {
          acc[a][b] = mfma32_bf16(am[a], bm, acc[a][b]);
          acc[a][b] = mfma32_bf16(al[a], bh, acc[a][b]);
          acc[a][b] = mfma32_bf16(ah[a], bl, acc[a][b]);
          acc[a][b] = mfma32_bf16(am[a], bh, acc[a][b]);
          acc[a][b] = mfma32_bf16(ah[a], bm, acc[a][b]);
          acc[a][b] = mfma32_bf16(ah[a], bh, acc[a][b]);
        }
      }
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
        const int pi = ptile * PT + pbase + 32 * a + 8 * (r >> 2) + 4 * kg + (r & 3);
        const int qi = qtile * QT + qbase + 32 * b + l32;
        if (pi < P) out[(size_t)pi * QTOT + qi] = acc[a][b][r];
      }
  if (ptile == 0) {
    // bias gradient: column sums of G; the two row octets of a column meet in LDS (fixed order)
    float* cs = (float*)smem_raw;  // [2][QT]; the last step's barrier has been passed by every wave
#pragma unroll
    for (int u = 0; u < GU; ++u)
      if (tid + 512 * u < 2 * QT) cs[goct[u] * QT + gcol[u]] = dbacc[u];
    __syncthreads();
    if (tid < QT) dbpart[(size_t)s * QTOT + qtile * QT + tid] = cs[tid] + cs[QT + tid];
  }
}

}  // namespace gfnx

namespace gfnx {

// Input-gradient product Out = (Gin W^T) . [act > 0] with the same three-piece arithmetic:
//   Out[i][p] = (sum_k Gin[i][k] * W[p][k]) * [act[i][p] > 0]  for the live rows i, written over the stored activation.
// W is the layer's own weight matrix, row-major with ldw floats per row of which Kvalid are used (its rows are
// contiguous in k, which is what the B operand of the 32 x 32 x 16 instruction wants: no transposed copy); the ReLU
// derivative comes from the recorded sign masks.
//
// The eight waves are CB = 8 / KH column blocks of 32 outputs x KH parts of the contraction, 128 indices each
// (KH = 2: contraction lengths up to 256, 128 outputs per workgroup; KH = 4: up to 512, 64 outputs per workgroup);
// a wave keeps the three pieces of its 32 x 128 slice of W in 96 registers for the whole kernel.  Tiles of 32
// transition rows go through LDS already split: every thread loads 8 consecutive values of a row (two 16-byte
// loads), splits them once, and writes three 16-byte pieces in operand order [piece][k octet][row]; the waves read
// their operands with 16-byte LDS loads.  NBUF = 2 (KH = 2): the tile after next is being loaded, the next one split
// and written, while the matrix cores work on the current one -- one barrier per tile (KH = 4 has LDS for one
// operand buffer: two barriers per tile).  The partial sums of the KH
// parts meet in a double-buffered LDS exchange after that barrier, in fixed order, and the part-0 waves store.
// grid = (row-tile workers (grid-stride), ceil(P / (32 CB))).  SCALE: Gin rows are multiplied by crow on load.
constexpr int kNt3Rows = 32;

template <int KH>
constexpr size_t gemm_nt3_lds_bytes() {
  constexpr int CB = 8 / KH, NBUF = KH == 2 ? 2 : 1, OCTS = 16 * KH;
  return (size_t)NBUF * 3 * OCTS * kNt3Rows * 16        // operand pieces
         + (size_t)2 * (KH - 1) * CB * 64 * 64            // partial-sum exchange
         + 8 * kNt3Rows * 4 + 8 * kNt3Rows * 4            // row ids and coefficients, a ring of eight tiles
         + 4 * kNt3Rows * 16 * 4;                         // sign-mask words, a ring of four tiles
}

template <int KH, bool SCALE>
__global__ __launch_bounds__(512) void gemm_nt3_kernel(const float* __restrict__ Gin, int ldgi, int K,
                                                       const float* __restrict__ W, int ldw, int Kvalid,
                                                       float* __restrict__ ActOut, int ldo, int P,
                                                       const unsigned long long* __restrict__ mask, int MW,
                                                       const float* __restrict__ crow,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr) {
  constexpr int CB = 8 / KH, PT = 32 * CB, NBUF = KH == 2 ? 2 : 1, OCTS = 16 * KH, R = kNt3Rows;
  constexpr int U = OCTS * R / 512;  // (row, k octet) units per thread and tile: 2 (KH = 2) or 4
  extern __shared__ __align__(16) unsigned char smem_raw[];
  u32x4* AS = (u32x4*)smem_raw;                                   // [NBUF][3][OCTS][R]
  f32x16* XCH = (f32x16*)(AS + NBUF * 3 * OCTS * R);              // [2][KH - 1][CB][64]
  int* ridb = (int*)(XCH + 2 * (KH - 1) * CB * 64);               // [8][R]
  float* cfb = (float*)(ridb + 8 * R);                            // [8][R]
  uint32_t* MSb = (uint32_t*)(cfb + 8 * R);                       // [4][16 words][R]: the mask words, transposed
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cb = w % CB, kh = w / CB, kg = lane >> 5, l32 = lane & 31;
  const int n = hdr[kHdrNLive];
  const int tiles = (n + R - 1) / R;
  const int pl = 32 * cb + l32, pcol = blockIdx.y * PT + pl;
  const int mwords = 2 * MW;  // 32-bit mask words per row (at most 16)

  // ---- this wave's slice of W: pieces of W[pcol][128 kh + 16 step + 8 kg .. + 7], step = 0 .. 7
  u32x4 wh[8], wm[8], wl[8];
#pragma unroll
  for (int st = 0; st < 8; ++st) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int kk = 128 * kh + 16 * st + 8 * kg + k;
      v[k] = (kk < Kvalid && pcol < P) ? W[(size_t)pcol * ldw + kk] : 0.f;
    }
    split3x8(v, wh[st], wm[st], wl[st]);
  }

  // ---- loader roles: unit = (row, k octet), rows fastest so that the LDS writes of a wave are contiguous
  const int octs = K >> 3;  // octets that exist (K is a multiple of 16)
  f32x4 pre[U][2];
  uint32_t mpre = 0;
  int idreg = -1;
  float cfreg = 0.f;
  auto fetch_ids = [&](int tile) {  // threads 0 .. R-1
    if (tid < R) {
      const bool on = tile < tiles && tile * R + tid < n;
      idreg = on ? rows[tile * R + tid] : -1;
      if (SCALE) cfreg = on ? crow[tile * R + tid] : 0.f;
    }
  };
  auto load_rows = [&](const int* ids) {
    if (tid < R * 16) {  // sign-mask words of the tile: R rows x (up to) 16 words
      const int rr = ids[tid >> 4], wd = tid & 15;
      mpre = (rr >= 0 && wd < mwords) ? ((const uint32_t*)mask)[(uint64_t)(uint32_t)max(rr, 0) * (uint32_t)mwords + (uint32_t)wd] : 0u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = tid + 512 * u, row = i & (R - 1), oct = i / R;
      const int rr = ids[row];
      const uint64_t off = (uint64_t)(uint32_t)max(rr, 0) * (uint32_t)ldgi + (uint32_t)(8 * min(oct, octs - 1));
      pre[u][0] = *(const f32x4*)&Gin[off];
      pre[u][1] = *(const f32x4*)&Gin[off + 4];
    }
  };
  auto store_tile = [&](int buf, const int* ids, const float* cfs) {
    u32x4* dst = AS + buf * 3 * OCTS * R;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = tid + 512 * u, row = i & (R - 1), oct = i / R;
      const bool on = ids[row] >= 0 && oct < octs;
      const float c = SCALE ? cfs[row] : 1.f;
      float v[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        v[k] = on ? (SCALE ? pre[u][0][k] * c : pre[u][0][k]) : 0.f;
        v[4 + k] = on ? (SCALE ? pre[u][1][k] * c : pre[u][1][k]) : 0.f;
      }
      u32x4 ph, pm, pq;
      split3x8(v, ph, pm, pq);
      dst[(0 * OCTS + oct) * R + row] = ph;
      dst[(1 * OCTS + oct) * R + row] = pm;
      dst[(2 * OCTS + oct) * R + row] = pq;
    }
  };

  // Tile k of this workgroup is row tile blockIdx.x + k * gridDim.x.  Row ids, coefficients and mask words live in
  // LDS rings from the request of a tile's rows to its epilogue; the epilogue of a tile runs after that tile's
  // barrier, beside the next tile's writes, so the rings are one tile deeper than the look-ahead.
  const int t0 = blockIdx.x, dt = gridDim.x;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    fetch_ids(t0 + k * dt);
    if (tid < R) { ridb[R * k + tid] = idreg; cfb[R * k + tid] = cfreg; }
  }
  lds_barrier();
  load_rows(ridb);
  if (NBUF == 2) {
    store_tile(0, ridb, cfb);
    if (tid < R * 16) MSb[(tid & 15) * R + (tid >> 4)] = mpre;
    load_rows(ridb + R);
  }
  fetch_ids(t0 + 3 * dt);
  lds_barrier();
  int it = 0;
  for (int tile = t0; tile < tiles; tile += dt, ++it) {
    const int* rid = ridb + R * (it & 7);
    if (NBUF == 2) {
      // rows of tile it+1 (in registers) are split into the other buffer, rows of tile it+2 requested
      store_tile((it + 1) & 1, ridb + R * ((it + 1) & 7), cfb + R * ((it + 1) & 7));
      if (tid < R * 16) MSb[((it + 1) & 3) * R * 16 + (tid & 15) * R + (tid >> 4)] = mpre;
      if (tid < R) { ridb[R * ((it + 3) & 7) + tid] = idreg; cfb[R * ((it + 3) & 7) + tid] = cfreg; }
      load_rows(ridb + R * ((it + 2) & 7));
      fetch_ids(tile + 4 * dt);
    } else {
      // one buffer: split this tile's rows (in registers), then request the next tile's
      store_tile(0, rid, cfb + R * (it & 7));
      if (tid < R * 16) MSb[(it & 3) * R * 16 + (tid & 15) * R + (tid >> 4)] = mpre;
      if (tid < R) { ridb[R * ((it + 3) & 7) + tid] = idreg; cfb[R * ((it + 3) & 7) + tid] = cfreg; }
      lds_barrier();
      load_rows(ridb + R * ((it + 1) & 7));
      fetch_ids(tile + 4 * dt);
    }
    const u32x4* src = AS + (NBUF == 2 ? (it & 1) : 0) * 3 * OCTS * R;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    {
      // steps past the contraction length hold nothing (uniform); the operands of step st+1 are read before the six
      // matrix instructions of step st
      const int nst = min(8, max(0, (K - 128 * kh + 15) >> 4));
      const u32x4* ap = src + (16 * kh + kg) * R + l32;
      u32x4 ah = ap[0], am = ap[OCTS * R], al = ap[2 * OCTS * R];
#pragma unroll
      for (int st = 0; st < 8; ++st) {
        if (st < nst) {
          u32x4 nh = ah, nm = am, nl = al;
          if (st + 1 < nst) {
            nh = ap[2 * (st + 1) * R];
            nm = ap[(OCTS + 2 * (st + 1)) * R];
            nl = ap[(2 * OCTS + 2 * (st + 1)) * R];
          }
          acc = mfma32_bf16(am, wm[st], acc);  // smallest products first
          acc = mfma32_bf16(al, wh[st], acc);
          acc = mfma32_bf16(ah, wl[st], acc);
          acc = mfma32_bf16(am, wh[st], acc);
          acc = mfma32_bf16(ah, wm[st], acc);
          acc = mfma32_bf16(ah, wh[st], acc);
          ah = nh; am = nm; al = nl;
        }
      }
    }
    f32x16* xch = XCH + (size_t)(it & 1) * (KH - 1) * CB * 64;
    if (kh > 0) xch[((kh - 1) * CB + cb) * 64 + lane] = acc;
    lds_barrier();
    if (kh == 0) {
#pragma unroll
      for (int q = 0; q < KH - 1; ++q) acc += xch[(q * CB + cb) * 64 + lane];
      if (pcol < P) {
        // unit u = pcol: bit (u % 256) / 4 of the 64-bit word 4 (u / 256) + u % 4 of the row; the words of this
        // lane's column and the row ids come as four 16-byte reads each (rows 8 q + 4 kg .. + 3, q = 0 .. 3).
        // Only the last row tile holds padding rows (id -1): every other tile stores without a test.
        const int bitpos = (pcol & 255) >> 2;
        const int word32 = 2 * (4 * (pcol >> 8) + (pcol & 3)) + (bitpos >> 5);
        const uint32_t* MS = MSb + (it & 3) * R * 16 + word32 * R;
        const uint32_t rowbytes = (uint32_t)ldo * 4u;
        char* const colbase = (char*)(ActOut + pcol);
        auto store_rows = [&](auto all_rows) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int4 ids = *(const int4*)&rid[8 * q + 4 * kg];
            const int4 mw = *(const int4*)&MS[8 * q + 4 * kg];
            const int id4[4] = {ids.x, ids.y, ids.z, ids.w};
            const int mw4[4] = {mw.x, mw.y, mw.z, mw.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              // all ones where the unit was active
              const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe(mw4[k], bitpos & 31, 1);
              const float av = acc[4 * q + k];  // (a copy: the cast below must not see the vector element itself)
              const float v = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, av) & keep);
              float* dst = (float*)(colbase + (uint64_t)(uint32_t)id4[k] * rowbytes);
              if (decltype(all_rows)::value || id4[k] >= 0) *dst = v;
            }
          }
        };
        if ((tile + 1) * R <= n)
          store_rows(std::true_type{});
        else
          store_rows(std::false_type{});
      }
    }
  }
}

// ---- Input-gradient product over a contraction of many pages of 256 (the logit layer of the paged rollout):
//   Out[i][p] = (sum_k crow[i] * Gin[i][k] * W[p][k]) * [act[i][p] > 0],  k = 0 .. 256 * pages - 1.
// Same three-piece arithmetic and the same wave roles as gemm_nt3_kernel<2> (4 column blocks of 32 outputs x 2 halves
// of a page), but the partial sums stay in registers across the pages: a workgroup takes a group of two 32-row tiles
// (two accumulators per wave: four would not leave registers for the slice), and for each page loads its slice of W once -- already cut into pieces and laid out in
// register order by split_w_pages_kernel, 1 KiB per wave and load -- and runs the tiles of the group against it.  The slice
// of the next page replaces the current one step by step during the last tile of the page, so its loads are in
// flight under the matrix work.  Tiles of Gin go through LDS as in gemm_nt3_kernel (two buffers, one barrier per
// tile); the two halves of the contraction meet once per group, in the epilogue.
// grid = (group workers (grid-stride), ceil(P / 128)): with a worker count that is a multiple of eight the column
// tiles of one group run on the same XCD (workgroups are dealt to the XCDs round-robin by their linear index), so a
// tile of Gin comes from HBM once and from that XCD's L2 cache for the other column tiles.
constexpr int kNt3pTiles = 2;

// Wsplit[(((ctile * pages + page) * 8 + wave) * 8 + step) * 3 + piece][lane]: pieces of
// W[128 ctile + 32 (wave % 4) + lane % 32][256 page + 128 (wave / 4) + 16 step + 8 (lane / 32) .. + 7].
// One workgroup of 512 threads per (page, ctile).
__global__ __launch_bounds__(512) void split_w_pages_kernel(const float* __restrict__ W, int ldw, int P, int pages,
                                                            u32x4* __restrict__ Wsplit) {
  const int page = blockIdx.x, ctile = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cb = w & 3, kh = w >> 2, kg = lane >> 5, l32 = lane & 31;
  const int pcol = 128 * ctile + 32 * cb + l32;
  u32x4* dst = Wsplit + ((size_t)(ctile * pages + page) * 8 + w) * 8 * 3 * 64 + lane;
#pragma unroll
  for (int st = 0; st < 8; ++st) {
    float v[8];
    const int k0 = 256 * page + 128 * kh + 16 * st + 8 * kg;
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = pcol < P ? W[(size_t)pcol * ldw + k0 + k] : 0.f;
    u32x4 ph, pm, pl;
    split3x8(v, ph, pm, pl);
    dst[(st * 3 + 0) * 64] = ph;
    dst[(st * 3 + 1) * 64] = pm;
    dst[(st * 3 + 2) * 64] = pl;
  }
}

constexpr size_t gemm_nt3p_lds_bytes() {
  return (size_t)2 * 3 * 32 * kNt3Rows * 16          // operand pieces of two tiles
         + (size_t)4 * 64 * 64                         // partial-sum exchange
         + kNt3pTiles * kNt3Rows * 8;                  // row ids and coefficients of the group
}

__global__ __launch_bounds__(512) void gemm_nt3p_kernel(const float* __restrict__ Gin, int ldgi, int pages,
                                                        const u32x4* __restrict__ Wsplit,
                                                        float* __restrict__ ActOut, int ldo, int P,
                                                        const unsigned long long* __restrict__ mask, int MW,
                                                        const float* __restrict__ crow,
                                                        const int* __restrict__ rows, const int* __restrict__ hdr) {
  constexpr int CB = 4, OCTS = 32, R = kNt3Rows, TG = kNt3pTiles;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  u32x4* AS = (u32x4*)smem_raw;                                   // [2][3][OCTS][R]
  f32x16* XCH = (f32x16*)(AS + 2 * 3 * OCTS * R);                 // [CB][64]
  int* gid = (int*)(XCH + CB * 64);                               // [TG * R] row ids of the group (-1: no row)
  float* gcf = (float*)(gid + TG * R);                            // [TG * R] their coefficients
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cb = w % CB, kh = w / CB, kg = lane >> 5, l32 = lane & 31;
  const int n = hdr[kHdrNLive];
  const int groups = (n + TG * R - 1) / (TG * R);
  const int ctile = blockIdx.y, worker = blockIdx.x, workers = gridDim.x;
  const int pcol = ctile * 128 + 32 * cb + l32;
  const int mwords = 2 * MW;
  const u32x4* wsrc = Wsplit + ((size_t)ctile * pages * 8 + w) * 8 * 3 * 64 + lane;  // + page * 8 * 8 * 3 * 64
  const size_t wpage = (size_t)8 * 8 * 3 * 64;
  const int S = pages * TG;  // tiles in the sequence of a group: page-major, the group's four row tiles within a page

  for (int grp = worker; grp < groups; grp += workers) {
    // ---- the group's rows
    if (tid < TG * R) {
      const int li = grp * TG * R + tid;
      gid[tid] = li < n ? rows[li] : -1;
      gcf[tid] = li < n ? crow[li] : 0.f;
    }
    lds_barrier();
    // loader: unit u of this thread = (row, k octet) of a tile, rows fastest
    f32x4 pre[2][2];
    auto load_rows = [&](int s) {  // tile s of the sequence: page s / TG, row tile s % TG
      const int page = s / TG, g = s - page * TG;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int i = tid + 512 * u, row = i & (R - 1), oct = i >> 5;
        const int rr = gid[g * R + row];
        const uint64_t off = (uint64_t)(uint32_t)max(rr, 0) * (uint32_t)ldgi + (uint32_t)(256 * page + 8 * oct);
        pre[u][0] = *(const f32x4*)&Gin[off];
        pre[u][1] = *(const f32x4*)&Gin[off + 4];
      }
    };
    auto store_tile = [&](int buf, int s) {
      const int g = s % TG;
      u32x4* dst = AS + buf * 3 * OCTS * R;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int i = tid + 512 * u, row = i & (R - 1), oct = i >> 5;
        const bool on = gid[g * R + row] >= 0;
        const float c = gcf[g * R + row];
        float v[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          v[k] = on ? pre[u][0][k] * c : 0.f;
          v[4 + k] = on ? pre[u][1][k] * c : 0.f;
        }
        u32x4 ph, pm, pq;
        split3x8(v, ph, pm, pq);
        dst[(0 * OCTS + oct) * R + row] = ph;
        dst[(1 * OCTS + oct) * R + row] = pm;
        dst[(2 * OCTS + oct) * R + row] = pq;
      }
    };

    u32x4 wh[8], wm[8], wl[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      wh[st] = wsrc[(st * 3 + 0) * 64];
      wm[st] = wsrc[(st * 3 + 1) * 64];
      wl[st] = wsrc[(st * 3 + 2) * 64];
    }
    f32x16 acc[TG];
#pragma unroll
    for (int g = 0; g < TG; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[g][r] = 0.f;

    load_rows(0);
    store_tile(0, 0);
    if (S > 1) load_rows(1);
    lds_barrier();

    for (int page = 0; page < pages; ++page) {
      const bool more_pages = page + 1 < pages;
      const u32x4* wnext = wsrc + (size_t)(page + 1) * wpage;
#pragma unroll
      for (int g = 0; g < TG; ++g) {
        const int s = page * TG + g;
        // the tile after this one (in registers) is cut into the other buffer, the one after that requested
        if (s + 1 < S) store_tile((s + 1) & 1, s + 1);
        if (s + 2 < S) load_rows(s + 2);
        const u32x4* ap = AS + (s & 1) * 3 * OCTS * R + (16 * kh + kg) * R + l32;
        u32x4 ah = ap[0], am = ap[OCTS * R], al = ap[2 * OCTS * R];
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          u32x4 nh = ah, nm = am, nl = al;
          if (st + 1 < 8) {
            nh = ap[2 * (st + 1) * R];
            nm = ap[(OCTS + 2 * (st + 1)) * R];
            nl = ap[(2 * OCTS + 2 * (st + 1)) * R];
          }
          acc[g] = mfma32_bf16(am, wm[st], acc[g]);  // smallest products first
          acc[g] = mfma32_bf16(al, wh[st], acc[g]);
          acc[g] = mfma32_bf16(ah, wl[st], acc[g]);
          acc[g] = mfma32_bf16(am, wh[st], acc[g]);
          acc[g] = mfma32_bf16(ah, wm[st], acc[g]);
          acc[g] = mfma32_bf16(ah, wh[st], acc[g]);
          if (g == TG - 1 && more_pages) {  // this step's slice of W is done with for this page: the next page's
            asm volatile("" ::: "memory");  // (requested here, not earlier: the registers are in use until now)
            wh[st] = wnext[(st * 3 + 0) * 64];
            wm[st] = wnext[(st * 3 + 1) * 64];
            wl[st] = wnext[(st * 3 + 2) * 64];
          }
          ah = nh; am = nm; al = nl;
        }
        lds_barrier();
      }
    }

    // ---- epilogue: the two halves of the contraction meet, mask, store; one tile at a time
    const int bitpos = (pcol & 255) >> 2;
    const int word32 = 2 * (4 * (pcol >> 8) + (pcol & 3)) + (bitpos >> 5);
#pragma unroll
    for (int g = 0; g < TG; ++g) {
      if (kh > 0) XCH[cb * 64 + lane] = acc[g];
      lds_barrier();
      if (kh == 0 && pcol < P) {
        const f32x16 other = XCH[cb * 64 + lane];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int id = gid[g * R + 8 * (r >> 2) + 4 * kg + (r & 3)];
          if (id >= 0) {
            const uint32_t mw = ((const uint32_t*)mask)[(uint64_t)(uint32_t)id * (uint32_t)mwords + (uint32_t)word32];
            const float a = acc[g][r] + other[r];
            ActOut[(uint64_t)(uint32_t)id * (uint32_t)ldo + (uint32_t)pcol] = ((mw >> (bitpos & 31)) & 1u) ? a : 0.f;
          }
        }
      }
      lds_barrier();
    }
  }
}

}  // namespace gfnx

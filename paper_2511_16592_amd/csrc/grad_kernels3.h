// Layer-1 weight gradient dW1 = onehot(s)^T G1 on the bf16 matrix cores.
//
// The left operand is a one-hot matrix (entries 0 or 1: exact in bf16), rebuilt from the state bytes the rollout
// recorded.  The right operand G1 is binary32; each value is cut into three bf16 pieces of 8 significant bits
// (g = hi + mid + lo exactly, by truncation), and the three products are accumulated in binary32 by the matrix
// core.  Every product is exact, so the result is a binary32-accumulated sum of the selected G1 rows, as the
// binary32 contraction gave, at a sixth of its matrix-core time (three bf16 instructions at sixteen times the rate).
//
// One workgroup = 8 waves; wave w owns output columns 32w .. 32w+31 for all (up to 256) one-hot columns: eight
// 32 x 32 accumulators.  Transition rows go through in rounds of 64 (four steps of 16 contraction rows):
//   - the one-hot operand of a round is built in LDS in MFMA A-operand order, [step][row-octet][column][8 x bf16];
//   - each lane fetches its G1 values (its column, 8 rows per step) straight from global memory, one step ahead;
//     a row of G1 is read by exactly one wave per 32 columns, so there is nothing to share through LDS.
// The transitions are split over the workgroups exactly as gemm_tn3_kernel splits them, partial tiles and column
// sums (the bias gradient) have the same layout, and the same fixed-order reductions finish the job.
#pragma once
#include "gfnx_device.h"
#include "grad_kernels.h"
#include "grad_kernels2.h"

namespace gfnx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// D(32x32) += A(32x16) * B(16x32), bf16 inputs.  Lane l supplies A[i = l%32][k = 8*(l/32) .. +7] and
// B[k = 8*(l/32) .. +7][j = l%32]; D as for mfma32.
__device__ __forceinline__ f32x16 mfma32_bf16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr int kDw1Round = 64;  // transition rows per round

// XSRC 1 (grid):  one-hot column p = H*i + x is 1 iff coordinate i equals x;
// XSRC 2 (Ising): column p = 2*site + s is 1 iff the site holds spin 2s-1 (the "unassigned" rows follow from the
//                 column sums, see reduce_dw1_ising_kernel).
// G: rows of ldg floats; blockIdx.y selects a tile of 256 of its columns; part: [S][P][QTOT]; dbpart: [S][QTOT];
// QTOT = 256 * gridDim.y.
template <int XSRC>
__global__ __launch_bounds__(512) void dw1_onehot_kernel(const float* __restrict__ G, int ldg,
                                                         const int* __restrict__ rows, const int* __restrict__ hdr,
                                                         const uint8_t* __restrict__ sbuf, int SB, int envH, int P,
                                                         int QTOT, float* __restrict__ part,
                                                         float* __restrict__ dbpart) {
  constexpr int R = kDw1Round;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  int* ids = (int*)smem_raw;                              // [3][R] row ids of three consecutive rounds
  unsigned char* SBs = smem_raw + 3 * R * 4;              // [R][SB] state bytes of the round being built
  u32x4* XSb = (u32x4*)(SBs + R * 112);                   // [2][4 steps][2 octets][256 columns] x (8 bf16)
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int s = blockIdx.x, S = gridDim.x;
  const int n = hdr[kHdrNLive];
  const int chunks = (n + 31) / 32;
  const int per = split_chunks_per_part(chunks, S);
  const int c0 = s * per, c1 = min(chunks, c0 + per);
  if (c0 >= c1) return;  // parts beyond the live transitions write nothing; the reduction skips them too
  const int row0 = 32 * c0, row1 = min(n, 32 * c1);      // this part's slice of the row list
  const int rounds = (row1 - row0 + R - 1) / R;
  const int PB = (P + 31) >> 5;                          // 32-column blocks of the one-hot operand in use
  const int q = 256 * blockIdx.y + 32 * w + (lane & 31), kg = lane >> 5;
  const bool qok = q < ldg;

  f32x16 acc[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  float dbacc = 0.f;

  // ---- per-thread roles
  // row ids: threads 0..63 fetch one id of a round
  auto fetch_id = [&](int round) -> int {
    const int li = row0 + round * R + tid;
    return (tid < R && round < rounds && li < row1) ? rows[li] : -1;
  };
  // state bytes: 16-byte pieces, SB/16 per row
  const int spr = SB >> 4;
  const int srow = tid / spr, spart = tid - srow * spr;
  auto fetch_state = [&](const int* idb) -> uint4 {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (srow < R) {
      const int id = idb[srow];
      if (id >= 0) v = *(const uint4*)&sbuf[(size_t)id * SB + 16 * spart];
    }
    return v;
  };
  // one-hot build: column p, row octet `oct` of every step
  const int p = tid & 255, oct = tid >> 8;
  int sdim, want;
  if (XSRC == 1) { sdim = p / envH; want = p - sdim * envH; }
  else { sdim = p >> 1; want = (p & 1) ? 1 : 255; }
  if (p >= P) { sdim = 0; want = 256; }  // never matches a byte
  auto build = [&](int buf) {
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      const unsigned char* src = SBs + (16 * step + 8 * oct) * SB + sdim;
      uint32_t b[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) b[k] = ((int)src[k * SB] == want) ? 0x3F80u : 0u;  // bf16(1.0) or 0
      u32x4 v;
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = b[2 * k] | (b[2 * k + 1] << 16);
      XSb[((buf * 4 + step) * 2 + oct) * 256 + p] = v;
    }
  };
  // this lane's G values for one step: rows 16*step + 8*kg .. +7 of the round, column q
  auto load_g = [&](const int* idb, int step, float g[8]) {
    const int4 i0 = *(const int4*)&idb[16 * step + 8 * kg], i1 = *(const int4*)&idb[16 * step + 8 * kg + 4];
    const int id[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
    for (int k = 0; k < 8; ++k) g[k] = (id[k] >= 0 && qok) ? G[(size_t)id[k] * ldg + q] : 0.f;
  };

  // ---- prologue: ids of rounds 0 and 1, state of round 0
  int idreg = fetch_id(0);
  if (tid < R) ids[tid] = idreg;
  lds_barrier();
  uint4 streg = fetch_state(ids);
  idreg = fetch_id(1);
  // the G values are requested two steps before their use
  float gn[8], gn2[8];
  load_g(ids, 0, gn);
  load_g(ids, 1, gn2);

  for (int it = 0; it < rounds; ++it) {
    const int* idb = ids + R * (it % 3);
    int* idb_next = ids + R * ((it + 1) % 3);
    if (srow < R) *(uint4*)&SBs[srow * SB + 16 * spart] = streg;
    if (tid < R) idb_next[tid] = idreg;
    lds_barrier();
    build(it & 1);
    streg = fetch_state(idb_next);  // in flight during this round's matrix work
    idreg = fetch_id(it + 2);
    lds_barrier();
    const u32x4* xa = XSb + (size_t)((it & 1) * 4) * 2 * 256 + kg * 256 + (lane & 31);
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      float g[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) { g[k] = gn[k]; gn[k] = gn2[k]; }
      if (step < 2) load_g(idb, step + 2, gn2);
      else load_g(idb_next, step - 2, gn2);  // first steps of the next round (ids of an absent round are all -1)
      // three bf16 pieces per value, packed in contraction order
      u32x4 bh, bm, bl;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        uint32_t h[2], m[2], l[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float x = g[2 * k + u];
          dbacc += x;
          h[u] = __builtin_bit_cast(uint32_t, x) & 0xFFFF0000u;
          const float r1 = x - __builtin_bit_cast(float, h[u]);
          m[u] = __builtin_bit_cast(uint32_t, r1) & 0xFFFF0000u;
          const float r2 = r1 - __builtin_bit_cast(float, m[u]);
          l[u] = __builtin_bit_cast(uint32_t, r2);
        }
        bh[k] = (h[0] >> 16) | h[1];
        bm[k] = (m[0] >> 16) | m[1];
        bl[k] = (l[0] >> 16) | (l[1] & 0xFFFF0000u);
      }
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        if (a < PB) {
          const u32x4 av = xa[(size_t)step * 2 * 256 + 32 * a];
          acc[a] = mfma32_bf16(av, bh, acc[a]);
          acc[a] = mfma32_bf16(av, bm, acc[a]);
          acc[a] = mfma32_bf16(av, bl, acc[a]);
        }
      }
    }
  }

  float* out = part + (size_t)s * P * QTOT;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int pi = 32 * a + 8 * (r >> 2) + 4 * kg + (r & 3);
      if (pi < P) out[(size_t)pi * QTOT + q] = acc[a][r];
    }
  dbacc += __shfl_xor(dbacc, 32);
  if (kg == 0) dbpart[(size_t)s * QTOT + q] = dbacc;
}

inline size_t dw1_onehot_lds_bytes() { return 3 * kDw1Round * 4 + kDw1Round * 112 + 2 * 4 * 2 * 256 * 16; }

// Backward pass of the logit layer for narrow action spaces (at most 16 logits, 256 hidden units), one sweep
// over the live transitions instead of two GEMM kernels whose contraction / output width would be 16:
//   g3 = c_b * e (16 values), dW3 += h2^T g3, db3 += g3, G2 = (W3 g3) . [h2 > 0] written over h2.
// A wave takes one transition at a time (eight in flight): lane l owns hidden units 4l .. 4l+3, i.e. 16 bytes of
// the 1 KiB row it reads and writes, its 4 x 16 slice of W3 and a 4 x 16 accumulator of dW3 in registers.  The
// work is HBM-bound (read h2, write G2: 2 KiB per transition); the 128 multiply-adds per lane hide under it.
// Transitions are split over the workgroups as in gemm_tn3_kernel and the partial tiles / column sums have its
// layout (part[s][unit][QTOT], dbpart[s][QTOT]), so the same reduction finishes dW3 and db3.
// crow[i] is the coefficient 2 delta_b / B of live transition i.
constexpr int kNarrowInFlight = 8;
constexpr int kNarrowLdsBytes = 8 * 16 * 64 * 16;
__global__ __launch_bounds__(512) void logit_bwd_narrow_kernel(float* __restrict__ h2buf, const float* __restrict__ ebuf,
                                                               const float* __restrict__ crow,
                                                               const float* __restrict__ W3, int A,
                                                               const int* __restrict__ rows, const int* __restrict__ hdr,
                                                               float* __restrict__ part, int QTOT,
                                                               float* __restrict__ dbpart) {
  constexpr int U = kNarrowInFlight;  // transitions in flight per wave
  extern __shared__ __align__(16) unsigned char smem_raw[];
  f32x4 (*red)[16][64] = (f32x4 (*)[16][64])smem_raw;  // [wave][logit][lane]: 4 units each; 128 KiB
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int s = blockIdx.x, S = gridDim.x;
  const int n = hdr[kHdrNLive];
  const int chunks = (n + 31) / 32;
  const int per = split_chunks_per_part(chunks, S);
  const int c0 = s * per, c1 = min(chunks, c0 + per);
  if (c0 >= c1) return;
  const int row0 = 32 * c0, row1 = min(n, 32 * c1);

  float w3r[4][16], acc[4][16];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      w3r[j][k] = k < A ? W3[(size_t)(4 * lane + j) * A + k] : 0.f;
      acc[j][k] = 0.f;
    }
  float dbl = 0.f;  // lanes 0..15: column sum of g3 for logit `lane`

  const int wu = __builtin_amdgcn_readfirstlane(w);
  for (int base = row0 + wu * U; base < row1; base += 8 * U) {
    // row id and coefficient are the same for every lane (scalar loads); per lane the 16 bytes of h2 and one value
    // of e: lane l holds e[l % 16], scaled into g3[l % 16] once the data is there, and the sixteen values reach the
    // multiply-adds as scalar operands read from lanes 0..15.  Little state per transition, so eight are in flight per
    // wave: the sweep is bound by HBM latency x bytes in flight.
    int id[U];
    float c[U], el[U];
    f32x4 h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int li = base + u;
      id[u] = li < row1 ? rows[li] : -1;
      c[u] = li < row1 ? crow[li] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t r = (size_t)(id[u] < 0 ? 0 : id[u]);
      h[u] = *(const f32x4*)&h2buf[r * 256 + 4 * lane];
      el[u] = ebuf[r * 16 + (lane & 15)];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (id[u] < 0) continue;  // uniform: the row index does not depend on the lane
      const float gl = c[u] * el[u];
      float g3[16];
#pragma unroll
      for (int k = 0; k < 16; ++k)
        g3[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, gl), k));
      if (lane < 16) dbl += gl;
      f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          acc[j][k] = __builtin_fmaf(h[u][j], g3[k], acc[j][k]);
          t[j] = __builtin_fmaf(w3r[j][k], g3[k], t[j]);
        }
      // ReLU derivative from the activation itself: it is still in hand before G2 goes over it
#pragma unroll
      for (int j = 0; j < 4; ++j) t[j] = h[u][j] > 0.f ? t[j] : 0.f;
      *(f32x4*)&h2buf[(size_t)id[u] * 256 + 4 * lane] = t;
    }
  }

  // fixed-order sum over the eight waves, then the partial tile of this workgroup
#pragma unroll
  for (int k = 0; k < 16; ++k) red[w][k][lane] = (f32x4){acc[0][k], acc[1][k], acc[2][k], acc[3][k]};
  __syncthreads();
  float* out = part + (size_t)s * 256 * QTOT;
  for (int i = tid; i < 16 * 64; i += 512) {
    const int k = i >> 6, l = i & 63;
    f32x4 v = red[0][k][l];
#pragma unroll
    for (int ww = 1; ww < 8; ++ww) v += red[ww][k][l];
#pragma unroll
    for (int j = 0; j < 4; ++j) out[(size_t)(4 * l + j) * QTOT + k] = v[j];
  }
  __syncthreads();
  float* dbs = (float*)&red[0][0][0];
  if (lane < 16) dbs[w * 16 + lane] = dbl;
  __syncthreads();
  if (tid < QTOT) {
    float v = 0.f;
    if (tid < 16)
#pragma unroll
      for (int ww = 0; ww < 8; ++ww) v += dbs[ww * 16 + tid];
    dbpart[(size_t)s * QTOT + tid] = v;
  }
}

}  // namespace gfnx

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
// The transitions are split over the workgroups exactly as gemm_tn2_kernel splits them, partial tiles and column
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
// G: rows of ldg floats (ldg <= 256 columns used); part: [S][P][QTOT = 256]; dbpart: [S][256].
template <int XSRC>
__global__ __launch_bounds__(512) void dw1_onehot_kernel(const float* __restrict__ G, int ldg,
                                                         const int* __restrict__ rows, const int* __restrict__ hdr,
                                                         const uint8_t* __restrict__ sbuf, int SB, int envH, int P,
                                                         float* __restrict__ part, float* __restrict__ dbpart) {
  constexpr int R = kDw1Round, QTOT = 256;
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
  const int q = 32 * w + (lane & 31), kg = lane >> 5;
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
  float gn[8];
  load_g(ids, 0, gn);

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
      for (int k = 0; k < 8; ++k) g[k] = gn[k];
      if (step < 3) load_g(idb, step + 1, gn);
      else load_g(idb_next, 0, gn);  // first step of the next round (ids of an absent round are all -1)
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

}  // namespace gfnx

// Gradient-pass kernels for hidden widths up to 256 (one workgroup covers a whole 256-wide operand).
//
//   gemm_tn2_kernel   dW = X^T G over the live transitions: 8 waves hold a (up to) 256 x 256 accumulator tile
//                     in registers, transition rows are gathered through the row list in chunks of 32, staged
//                     in LDS, the next chunk's global loads are in flight while the matrix cores work;
//                     column sums of G (the bias gradient) ride along.
//   gemm_nt2_kernel   Out = (G W^T) . [act > 0]: each wave keeps a 32-column slice of W in registers as the
//                     MFMA B operand for the whole kernel; tiles of 64 transition rows stream through LDS.
//   dw1_lds_kernel    layer-1 weight gradient: per-trajectory segment sums accumulated in an LDS copy of a
//                     feature slice of dW1 (LDS float atomics), flushed once per workgroup.
//   reduce2_kernel    fixed-order sum of the split partials.
// With SCALE the G operand is (2 delta_b / B) * e, formed while the rows are loaded, so the logit-gradient rows
// are never rewritten in HBM.
#pragma once
#include "gfnx_device.h"
#include "grad_kernels.h"

namespace gfnx {

template <int WP, int WQ, int PBW, int QBW, bool SCALE>
__global__ __launch_bounds__(512) void gemm_tn2_kernel(const float* __restrict__ X, int ldx, int P,
                                                       const float* __restrict__ G, int ldg,
                                                       const float* __restrict__ coef, int B,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr,
                                                       int QTOT, float* __restrict__ part,
                                                       float* __restrict__ dbpart) {
  constexpr int PT = WP * PBW * 32, QT = WQ * QBW * 32, KC = 32;
  constexpr int XV = KC * PT / 4 / 512, GV = (KC * QT / 4 + 511) / 512;  // f32x4 per thread per chunk
  static_assert(WP * WQ == 8, "eight waves");
  extern __shared__ float smem[];
  float* XS = smem;             // [KC][PT]
  float* GS = smem + KC * PT;   // [KC][QT]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ptile = blockIdx.x, qtile = blockIdx.y, s = blockIdx.z, S = gridDim.z;
  const int n = hdr[kHdrNLive];
  const int chunks = (n + KC - 1) / KC;
  const int per = (chunks + S - 1) / S;
  const int c0 = s * per, c1 = min(chunks, c0 + per);
  const int pbase = (w / WQ) * PBW * 32, qbase = (w % WQ) * QBW * 32;

  f32x16 acc[PBW][QBW];
#pragma unroll
  for (int a = 0; a < PBW; ++a)
#pragma unroll
    for (int b = 0; b < QBW; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  float dbacc = 0.f;

  f32x4 xr[XV], gr[GV];
  auto load_chunk = [&](int c) {
#pragma unroll
    for (int m = 0; m < XV; ++m) {
      const int i = tid + 512 * m;
      const int r = i / (PT / 4), c4 = i % (PT / 4);
      const int li = c * KC + r;
      xr[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (li < n && ptile * PT + 4 * c4 < P) xr[m] = *(const f32x4*)&X[(size_t)rows[li] * ldx + ptile * PT + 4 * c4];
    }
#pragma unroll
    for (int m = 0; m < GV; ++m) {
      const int i = tid + 512 * m;
      const int r = i / (QT / 4), c4 = i % (QT / 4);
      const int li = c * KC + r;
      const int col = qtile * QT + 4 * c4;
      gr[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (i < KC * QT / 4 && li < n && col < ldg) {
        const int rid = rows[li];
        f32x4 v = *(const f32x4*)&G[(size_t)rid * ldg + col];
        if (SCALE) v = v * coef[rid % B];
        gr[m] = v;
      }
    }
  };
  auto store_chunk = [&]() {
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

  if (c0 < c1) load_chunk(c0);
  for (int c = c0; c < c1; ++c) {
    store_chunk();
    lds_barrier();
    if (c + 1 < c1) load_chunk(c + 1);
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

// out[p*Q + q] = sum_s part[s][p][q], q < Q; four outputs per thread, eight partials in flight.
__global__ void reduce2_kernel(const float* __restrict__ part, int S, int P, int QTOT, int Q, float* __restrict__ out) {
  const int qv = QTOT >> 2;
  const size_t total = (size_t)P * qv;
  const size_t stride = (size_t)P * QTOT;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int p = (int)(i / qv), q4 = (int)(i % qv) * 4;
    if (q4 >= Q) continue;
    const float* src = part + (size_t)p * QTOT + q4;
    f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
    int s = 0;
    for (; s + 4 <= S; s += 4) {
      a0 += *(const f32x4*)&src[(size_t)s * stride];
      a1 += *(const f32x4*)&src[(size_t)(s + 1) * stride];
      a2 += *(const f32x4*)&src[(size_t)(s + 2) * stride];
      a3 += *(const f32x4*)&src[(size_t)(s + 3) * stride];
    }
    for (; s < S; ++s) a0 += *(const f32x4*)&src[(size_t)s * stride];
    const f32x4 v = (a0 + a1) + (a2 + a3);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (q4 + k < Q) out[(size_t)p * Q + q4 + k] = v[k];
  }
}

// For each live row i: Out[i][p] = (sum_q Gin[i][q] * W[p][q]) * [Out[i][p] > 0], in place over the stored
// activation; contraction length K <= 256 (rows of Gin hold K floats, W rows hold Kvalid <= K).
// grid = (row-tile workers (grid-stride), ceil(P/256)); 8 waves, wave w owns output columns 32w .. 32w+31.
template <bool SCALE>
__global__ __launch_bounds__(512) void gemm_nt2_kernel(const float* __restrict__ Gin, int ldgi, int K,
                                                       const float* __restrict__ W, int Kvalid,
                                                       float* __restrict__ ActOut, int ldo, int P,
                                                       const float* __restrict__ coef, int B,
                                                       const int* __restrict__ rows, const int* __restrict__ hdr) {
  constexpr int KP = 258;  // LDS row pitch in floats: even (8-byte reads) and 2 mod 32 (conflict-free rows)
  extern __shared__ float smem[];
  float* GS = smem;                    // [64][KP]
  int* rid = (int*)(smem + 64 * KP);   // [64]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = hdr[kHdrNLive];
  const int tiles = (n + 63) >> 6;
  const int pcol = blockIdx.y * 256 + 32 * w + (lane & 31);
  const int kk = lane >> 5;

  // B operand: step s consumes contraction index q = 4*(s/2) + 2*kk + (s%2)
  float wreg[128];
#pragma unroll
  for (int s = 0; s < 128; ++s) {
    const int q = 4 * (s >> 1) + 2 * kk + (s & 1);
    wreg[s] = (q < Kvalid && pcol < P) ? W[(size_t)pcol * Kvalid + q] : 0.f;
  }

  const int kv = K >> 2;               // f32x4 per row
  f32x4 pre[8];
  int my_rid[8];
  auto load_tile = [&](int tile) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;     // 64 rows x 64 quads
      const int r = i >> 6, c4 = i & 63;
      const int li = tile * 64 + r;
      pre[m] = (f32x4){0.f, 0.f, 0.f, 0.f};
      my_rid[m] = -1;
      if (li < n) {
        const int rr = rows[li];
        my_rid[m] = rr;
        if (c4 < kv) {
          f32x4 v = *(const f32x4*)&Gin[(size_t)rr * ldgi + 4 * c4];
          if (SCALE) v = v * coef[rr % B];
          pre[m] = v;
        }
      }
    }
  };

  int tile = blockIdx.x;
  if (tile < tiles) load_tile(tile);
  for (; tile < tiles; tile += gridDim.x) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = tid + 512 * m;
      const int r = i >> 6, c4 = i & 63;
      float* d = &GS[r * KP + 4 * c4];
      *(float2*)d = make_float2(pre[m].x, pre[m].y);
      *(float2*)(d + 2) = make_float2(pre[m].z, pre[m].w);
      if (c4 == 0) rid[r] = my_rid[m];
    }
    lds_barrier();
    if (tile + (int)gridDim.x < tiles) load_tile(tile + gridDim.x);
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    const float* g0 = &GS[(lane & 31) * KP + 2 * kk];
    const float* g1 = g0 + 32 * KP;
#pragma unroll
    for (int s2 = 0; s2 < 64; ++s2) {
      if (4 * s2 < K) {
        const float2 a0 = *(const float2*)&g0[4 * s2];
        const float2 a1 = *(const float2*)&g1[4 * s2];
        acc0 = mfma32(a0.x, wreg[2 * s2], acc0);
        acc1 = mfma32(a1.x, wreg[2 * s2], acc1);
        acc0 = mfma32(a0.y, wreg[2 * s2 + 1], acc0);
        acc1 = mfma32(a1.y, wreg[2 * s2 + 1], acc1);
      }
    }
    if (pcol < P) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 8 * (r >> 2) + 4 * kk + (r & 3);
        const int r0 = rid[i], r1 = rid[32 + i];
        if (r0 >= 0) {
          float* o = &ActOut[(size_t)r0 * ldo + pcol];
          *o = (*o > 0.f) ? acc0[r] : 0.f;
        }
        if (r1 >= 0) {
          float* o = &ActOut[(size_t)r1 * ldo + pcol];
          *o = (*o > 0.f) ? acc1[r] : 0.f;
        }
      }
    }
    lds_barrier();
  }
}

constexpr int kDw1Waves = 16;  // trajectories a workgroup of dw1_lds_kernel works on at a time

// Layer-1 weight gradient with an LDS-private copy of a 64-feature slice of dW1 (obs_dim rows).
// grid = (trajectory groups, H1/64); 1024 threads = 16 trajectories at a time x 64 features; the row bookkeeping
// of a trajectory (which one-hot row leaves / enters at each step) is rebuilt from its action bytes.
// Segment sums as in dw1_kernel: one running sum per grid coordinate, or prefix + suffix sweeps.
template <int ENV>
__global__ __launch_bounds__(1024) void dw1_lds_kernel(const Dw1Params p, int traj_per_group) {
  extern __shared__ float smem[];
  const EnvParams& e = p.env;
  const int rows_n = e.obs_dim;
  float* tab = smem;                                   // [obs_dim][64]
  int* rold = (int*)(smem + (size_t)rows_n * 64);      // [16][256]
  int* rnew = rold + kDw1Waves * 256;                  // [16][256]
  int* rend = rnew + kDw1Waves * 256;                  // [16][kMaxStateDim]
  int* meta = rend + kDw1Waves * kMaxStateDim;         // [16][4]: len, nend
  int8_t* st = (int8_t*)(meta + kDw1Waves * 4);        // [16][kMaxStateDim]
  const int tid = threadIdx.x, f = tid & 63, tq = tid >> 6;
  const int H1 = p.H1, B = p.B, f0 = blockIdx.y * 64;
  for (int i = tid; i < rows_n * 64; i += 1024) tab[i] = 0.f;
  float dbsum = 0.f;
  const int g0 = blockIdx.x * traj_per_group;
  for (int base = 0; base < traj_per_group; base += kDw1Waves) {
    const int b = g0 + base + tq;
    __syncthreads();
    // stage the action bytes of the four trajectories in LDS (rnew doubles as the staging area)
    int len_b = (b < B) ? p.length[b] : 0;
    len_b = len_b < 0 ? 0 : (len_b > e.max_steps ? e.max_steps : len_b);
    for (int t = f; t + 1 < len_b; t += 64) rnew[tq * 256 + t] = p.actions[(size_t)t * B + b];
    __syncthreads();
    if (f == 0) {
      const int len = len_b;
      int bad = 0;
      int8_t* s8 = st + tq * kMaxStateDim;
      for (int s = 0; s < e.state_dim; ++s) s8[s] = 0;
      for (int t = 0; t + 1 < len; ++t) {
        const int a = rnew[tq * 256 + t];
        if (ENV == 0 ? (a >= e.d || s8[a] >= e.H - 1) : (a >= e.n_actions)) { bad = 1; break; }
        if (ENV == 0) {
          rold[tq * 256 + t] = e.H * a + s8[a];
          rnew[tq * 256 + t] = a;
          s8[a] += 1;
        } else if (ENV == 1) {
          rold[tq * 256 + t] = ((1 << e.k_bits) + 1) * t + (1 << e.k_bits);
          rnew[tq * 256 + t] = ((1 << e.k_bits) + 1) * t + a;
          s8[t] = 1;
        } else {
          rold[tq * 256 + t] = 3 * (a >> 1) + 1;
          rnew[tq * 256 + t] = 3 * (a >> 1) + 1 + 2 * (a & 1) - 1;
          s8[a >> 1] = 1;
        }
      }
      int nend = 0;
      for (int s = 0; s < e.state_dim; ++s) {
        if (ENV == 0) rend[tq * kMaxStateDim + nend++] = e.H * s + s8[s];
        else if (ENV == 1) { if (!s8[s]) rend[tq * kMaxStateDim + nend++] = ((1 << e.k_bits) + 1) * s + (1 << e.k_bits); }
        else { if (!s8[s]) rend[tq * kMaxStateDim + nend++] = 3 * s + 1; }
      }
      meta[tq * 4 + 0] = bad ? 0 : len;
      meta[tq * 4 + 1] = nend;
    }
    __syncthreads();
    const int len = meta[tq * 4 + 0], nend = meta[tq * 4 + 1];
    if (len <= 0) continue;
    const float* g1 = p.g1 + (size_t)b * H1 + f0 + f;
    const size_t stride = (size_t)B * H1;
    const int* ro = rold + tq * 256;
    const int* rn = rnew + tq * 256;
    const int* re = rend + tq * kMaxStateDim;
    if (ENV == 0) {
      float acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      float total = 0.f;
      for (int t0 = 0; t0 < len; t0 += 8) {
        float gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) gv[u] = (t0 + u < len) ? g1[(t0 + u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u;
          if (t < len) {
            const float g = gv[u];
            total += g;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] += g;
            if (t + 1 < len) {
              const int a = rn[t];
              float v = 0.f;
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (i == a) { v = acc[i]; acc[i] = 0.f; }
              atomicAdd(&tab[ro[t] * 64 + f], v);
            }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (i < e.d) atomicAdd(&tab[re[i] * 64 + f], acc[i]);
      dbsum += total;
    } else {
      float P = 0.f;
      for (int t0 = 0; t0 < len; t0 += 8) {
        float gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) gv[u] = (t0 + u < len) ? g1[(t0 + u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u;
          if (t < len) {
            P += gv[u];
            if (t + 1 < len) atomicAdd(&tab[ro[t] * 64 + f], P);
          }
        }
      }
      for (int i = 0; i < nend; ++i) atomicAdd(&tab[re[i] * 64 + f], P);
      dbsum += P;
      float S = 0.f;
      for (int t0 = len - 1; t0 >= 1; t0 -= 8) {
        float gv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) gv[u] = (t0 - u >= 1) ? g1[(t0 - u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 - u;
          if (t >= 1) {
            S += gv[u];
            atomicAdd(&tab[rn[t - 1] * 64 + f], S);
          }
        }
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < rows_n * 64; i += 1024) {
    const float v = tab[i];
    if (v != 0.f) atomicAdd(&p.dW1[(size_t)(i >> 6) * H1 + f0 + (i & 63)], v);
  }
  atomicAdd(&p.db1[f0 + f], dbsum);
}

}  // namespace gfnx

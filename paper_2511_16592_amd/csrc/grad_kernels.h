// Gradient pass of the Trajectory-Balance loss over the transitions recorded by the rollout: bookkeeping kernels
// and the layer-1 fallback.
//
// The live transitions (t < length[b]) are listed in (t, b) order; every kernel of the pass works on that list,
// so padded steps cost nothing.  With coef_b = 2 delta_b / B the chain is
//   G3 = coef * (onehot(a) - p)                      (formed on load, never stored)
//   dW3 = H2^T G3, db3 = colsum G3                   (gemm_tn3_kernel, split over the transitions)
//   G2 = (G3 W3^T) . [h2 > 0]   written over h2      (gemm_nt3_kernel; both in logit_bwd_narrow_kernel for <= 16 logits)
//   dW2 = H1^T G2, db2 = colsum G2                   (gemm_tn3_kernel)
//   G1 = (G2 W2^T) . [h1 > 0]   written over h1      (gemm_nt3_kernel)
//   dW1, db1 from G1                                 (dw1_onehot_kernel; dw1_kernel below for wide one-hot inputs)
// This file: rows_kernel (residuals, loss, the list), adam_kernel (optimiser step), fill_kernel, dw1_kernel
// (per-trajectory segment sums with atomics).
#pragma once
#include "gfnx_device.h"

namespace gfnx {

constexpr int kHdrNLive = 0;    // header words (int32)
constexpr int kHdrCnt = 16;     // cnt[t] = number of trajectories longer than t, t < 256
constexpr int kHdrOff = 16 + 256;  // off[t] = first list position of step t
constexpr int kHdrWords = 16 + 512;

// Workgroup t lists the live transitions of step t in increasing b: rows[off[t] + rank] = t*B + b, and next to each
// the coefficient of its trajectory, crow[off[t] + rank] = 2 delta_b / B with the TB residual
// delta_b = log Z + log P_F - log R - log P_B.  Every workgroup derives the list offsets itself from the histogram
// of the lengths (B integers: cheaper than a launch of its own): cnt[u] = #{b : len_b > u} is a suffix sum of the
// histogram and off[u] a prefix sum of cnt, both taken by one wavefront with four entries per lane; workgroup 0 also
// writes them to the header for the kernels that follow, together with the loss (mean delta^2) and dloss/dlogZ
// (2 mean delta).  The list itself takes two sweeps over the lengths (count per wavefront, then write), one barrier
// between them.  T <= 256.
__global__ __launch_bounds__(1024) void rows_kernel(const int* __restrict__ length, const float* __restrict__ lpf,
                                                    const float* __restrict__ lpb, const float* __restrict__ logr,
                                                    float log_z, const float* __restrict__ log_z_dev, int B, int T,
                                                    float* __restrict__ loss, float* __restrict__ dlogz,
                                                    int* __restrict__ hdr, int* __restrict__ rows,
                                                    float* __restrict__ crow) {
  if (log_z_dev) log_z = *log_z_dev;  // log Z kept on the device (training loop) instead of passed by value
  __shared__ int hist[260];             // hist[l] = #{b : len_b = l}, l = 0 .. 256 (clamped to [0, T])
  __shared__ int cnts[256], offs[256];
  __shared__ float red2[16], red1[16];
  __shared__ int wsum[16];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  for (int i = tid; i < 260; i += 1024) hist[i] = 0;
  __syncthreads();
  float s2 = 0.f, s1 = 0.f;
  for (int b = tid; b < B; b += 1024) {
    if (t == 0) {
      const float delta = log_z + lpf[b] - logr[b] - lpb[b];
      s2 += delta * delta;
      s1 += delta;
    }
    int len = length[b];
    len = len < 0 ? 0 : (len > T ? T : len);
    atomicAdd(&hist[len], 1);
  }
  if (t == 0) {  // fixed-order sums: lanes of a wavefront by halving, then the sixteen wavefronts in order
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { s2 += __shfl_down(s2, o); s1 += __shfl_down(s1, o); }
    if (lane == 0) { red2[wv] = s2; red1[wv] = s1; }
  }
  __syncthreads();
  if (wv == 0) {
    // lane i owns steps u = 4i .. 4i+3: cnt[u] = sum_{l > u} hist[l], off[u] = sum_{v < u} cnt[v]
    int h[4], c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) h[k] = hist[4 * lane + k + 1];
    c[3] = h[3]; c[2] = h[2] + c[3]; c[1] = h[1] + c[2]; c[0] = h[0] + c[1];
    int above = c[0];  // inclusive suffix sum of the lane totals, then made exclusive
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_down(above, o);
      if (lane + o < 64) above += v;
    }
    above -= c[0];
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] += above;
    const int mine = c[0] + c[1] + c[2] + c[3];
    int before = mine;  // inclusive prefix sum of the lane totals, then made exclusive
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(before, o);
      if (lane >= o) before += v;
    }
    before -= mine;
    int run = before;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int u = 4 * lane + k;
      cnts[u] = c[k];
      offs[u] = run;
      if (t == 0 && u < T) { hdr[kHdrCnt + u] = c[k]; hdr[kHdrOff + u] = run; }
      run += c[k];
    }
    if (t == 0) {
      if (lane == 63) hdr[kHdrNLive] = run;  // all live transitions: the last lane's running total
      if (lane == 0) {
        float a2 = 0.f, a1 = 0.f;
        for (int k = 0; k < 16; ++k) { a2 += red2[k]; a1 += red1[k]; }
        *loss = a2 / (float)B;
        *dlogz = 2.f * a1 / (float)B;
      }
    }
  }
  __syncthreads();
  const int mycnt = cnts[t];
  if (mycnt == 0) return;
  // this workgroup's rows: wavefront w takes the b-range [w * per, (w + 1) * per), per a multiple of 64
  const int per = ((B + 15) / 16 + 63) & ~63;
  const int lo = wv * per, hi = min(B, lo + per);
  int mine = 0;
  for (int b = lo + lane; b < hi; b += 64) mine += length[b] > t ? 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  if (lane == 0) wsum[wv] = mine;
  __syncthreads();
  int pos = offs[t];
  for (int k = 0; k < wv; ++k) pos += wsum[k];
  for (int b0 = lo; b0 < hi; b0 += 64) {
    const int b = b0 + lane;
    const bool on = b < hi && length[b] > t;
    const unsigned long long bal = __ballot(on);
    if (on) {
      const int at = pos + __popcll(bal & ((1ull << lane) - 1ull));
      rows[at] = t * B + b;
      crow[at] = 2.f * (log_z + lpf[b] - logr[b] - lpb[b]) / (float)B;
    }
    pos += __popcll(bal);
  }
}

// Adam update (Kingma & Ba 2015, Algorithm 1) of up to kAdamMaxJobs tensors in one elementwise launch.  c1, c2 are
// the bias corrections 1 - beta1^t, 1 - beta2^t of this update.  Workgroup i serves 1024 consecutive elements of
// the tensor whose block range [first[j], first[j+1]) holds i, four per lane.  HBM-bound: 16 B read + 12 B written per parameter.
constexpr int kAdamMaxJobs = 8;
struct AdamJobs {
  float* theta[kAdamMaxJobs];
  const float* g[kAdamMaxJobs];
  float* m[kAdamMaxJobs];
  float* v[kAdamMaxJobs];
  unsigned n[kAdamMaxJobs];
  float lr[kAdamMaxJobs];
  int first[kAdamMaxJobs + 1];
  int jobs;
  float beta1, beta2, eps, c1, c2;
};

__device__ __forceinline__ void adam_one(float& theta, float g, float& m, float& v, float lr, const AdamJobs& a) {
  m = a.beta1 * m + (1.f - a.beta1) * g;
  v = a.beta2 * v + (1.f - a.beta2) * (g * g);
  theta = theta - lr * (m / a.c1) / (sqrtf(v / a.c2) + a.eps);
}

__global__ __launch_bounds__(256) void adam_kernel(AdamJobs a) {
  int j = 0;
  while (j + 1 < a.jobs && (int)blockIdx.x >= a.first[j + 1]) ++j;
  float* __restrict__ theta = a.theta[j];
  const float* __restrict__ g = a.g[j];
  float* __restrict__ m = a.m[j];
  float* __restrict__ v = a.v[j];
  const unsigned n = a.n[j];
  const float lr = a.lr[j];
  const unsigned i0 = ((unsigned)((int)blockIdx.x - a.first[j]) * 256u + threadIdx.x) * 4u;  // four elements per lane
  if (i0 >= n) return;
  const bool aligned = ((((uintptr_t)theta) | ((uintptr_t)g) | ((uintptr_t)m) | ((uintptr_t)v)) & 15) == 0;
  if (aligned && i0 + 4 <= n) {
    float4 t4 = *(const float4*)(theta + i0), m4 = *(const float4*)(m + i0), v4 = *(const float4*)(v + i0);
    const float4 g4 = *(const float4*)(g + i0);
    adam_one(t4.x, g4.x, m4.x, v4.x, lr, a);
    adam_one(t4.y, g4.y, m4.y, v4.y, lr, a);
    adam_one(t4.z, g4.z, m4.z, v4.z, lr, a);
    adam_one(t4.w, g4.w, m4.w, v4.w, lr, a);
    *(float4*)(theta + i0) = t4;
    *(float4*)(m + i0) = m4;
    *(float4*)(v + i0) = v4;
  } else {
    for (unsigned i = i0; i < n && i < i0 + 4; ++i) adam_one(theta[i], g[i], m[i], v[i], lr, a);
  }
}

__global__ void fill_kernel(float* __restrict__ p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

struct Dw1Params {
  EnvParams env;
  int H1, B;
  const uint8_t* actions;
  const uint16_t* actions16;  // used instead of `actions` when not null (more than 256 actions)
  const int* length;
  const int8_t* term;
  const float* g1;  // rows t*B + b, H1 floats
  float *dW1, *db1;
  int suffix_only;  // bit sequences: the "empty" rows and db1 come from the per-step column sums instead
};

// One workgroup per trajectory; dW1[r] += sum of g1_t over the steps t at which one-hot row r is active.
// A row is active on a contiguous run of steps, so no per-step scatter over all active rows is needed:
//   grid    one running sum per coordinate, flushed to row (i, x_i) when coordinate i is incremented;
//   bitseq (either scheme), Ising   a position has two phases: its "empty/unassigned" row is active up to the step that
//           fills it (a prefix sum of g1), the row of the value written is active afterwards (a suffix
//           sum, taken in a second sweep from the end).
// Only sums of like terms are formed (no differences of long prefix sums), the total is the bias gradient.
template <int ENV>
__global__ __launch_bounds__(256) void dw1_kernel(const Dw1Params p) {
  __shared__ int rold[256], rnew[256], rend[kMaxStateDim];
  __shared__ int nend;
  __shared__ int8_t st[kMaxStateDim];
  const EnvParams& e = p.env;
  const int b = blockIdx.x, tid = threadIdx.x, H1 = p.H1, B = p.B;
  int len = p.length[b];
  if (len <= 0) return;
  if (len > e.max_steps) len = e.max_steps;  // malformed input must not index out of bounds
  __shared__ int bad;
  if (tid == 0) {
    bad = 0;
    for (int s = 0; s < e.state_dim; ++s) st[s] = 0;
    for (int t = 0; t + 1 < len; ++t) {
      int a = p.actions16 ? (int)p.actions16[(size_t)t * B + b] : (int)p.actions[(size_t)t * B + b];
      if (ENV == 0 ? (a >= e.d || st[a] >= e.H - 1)
                   : (ENV == 3 ? (a >= e.n_actions || st[a >> e.k_bits]) : (a >= e.n_actions))) { bad = 1; break; }
      if (ENV == 0) {
        rold[t] = e.H * a + st[a];  // row left by this increment
        rnew[t] = a;                // coordinate whose running sum is flushed
        st[a] += 1;
      } else if (ENV == 1) {
        rold[t] = ((1 << e.k_bits) + 1) * t + (1 << e.k_bits);
        rnew[t] = ((1 << e.k_bits) + 1) * t + a;
        st[t] = 1;
      } else if (ENV == 3) {
        const int pos = a >> e.k_bits;
        rold[t] = ((1 << e.k_bits) + 1) * pos + (1 << e.k_bits);
        rnew[t] = ((1 << e.k_bits) + 1) * pos + (a & ((1 << e.k_bits) - 1));
        st[pos] = 1;
      } else {
        rold[t] = 3 * (a >> 1) + 1;
        rnew[t] = 3 * (a >> 1) + 1 + 2 * (a & 1) - 1;
        st[a >> 1] = 1;
      }
    }
    // rows still in their first phase at the last evaluated state s_{len-1}
    int n = 0;
    for (int s = 0; s < e.state_dim; ++s) {
      if (ENV == 0) rend[n++] = e.H * s + st[s];
      else if (ENV == 1 || ENV == 3) { if (!st[s]) rend[n++] = ((1 << e.k_bits) + 1) * s + (1 << e.k_bits); }
      else { if (!st[s]) rend[n++] = 3 * s + 1; }
    }
    nend = n;
  }
  __syncthreads();
  if (bad) return;  // an action that is impossible in its state: the trajectory contributes nothing
  for (int f = tid; f < H1; f += 256) {
    const float* g1 = p.g1 + (size_t)b * H1 + f;
    const size_t stride = (size_t)B * H1;
    if (ENV == 0) {
      float acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      float total = 0.f;
      for (int t = 0; t < len; ++t) {
        const float g = g1[t * stride];
        total += g;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] += g;
        if (t + 1 < len) {
          const int a = rnew[t];
          float v = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (i == a) { v = acc[i]; acc[i] = 0.f; }
          atomicAdd(&p.dW1[(size_t)rold[t] * H1 + f], v);
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (i < e.d) atomicAdd(&p.dW1[(size_t)rend[i] * H1 + f], acc[i]);
      atomicAdd(&p.db1[f], total);
    } else {
      if (!p.suffix_only) {
        float P = 0.f;
        for (int t = 0; t < len; ++t) {
          P += g1[t * stride];
          if (t + 1 < len) atomicAdd(&p.dW1[(size_t)rold[t] * H1 + f], P);
        }
        for (int i = 0; i < nend; ++i) atomicAdd(&p.dW1[(size_t)rend[i] * H1 + f], P);
        atomicAdd(&p.db1[f], P);
      }
      float S = 0.f;
      for (int t = len - 1; t >= 1; --t) {
        S += g1[t * stride];
        atomicAdd(&p.dW1[(size_t)rnew[t - 1] * H1 + f], S);
      }
    }
  }
}

// Bit sequences: every trajectory shares the same "empty" rows, so their gradient is not scattered per trajectory.
// The empty row of position s is active at step t' iff t' <= s, for every trajectory alive at t': its gradient is
// the sum over t' <= s of the column sums cs[t'] of G1 over the live rows of step t', and db1 is the sum of all.
//   colsum_steps_kernel  grid (steps, parts): partial column sums of a slab of one step's rows, added to cs[t]
//                        (cs zeroed before; at most `parts` atomics meet on an address)
//   bitseq_empty_rows_kernel  grid (positions): prefix over the steps, plain stores to dW1; block 0 also writes db1
__global__ __launch_bounds__(256) void colsum_steps_kernel(const float* __restrict__ g1, int H1,
                                                           const int* __restrict__ rows, const int* __restrict__ hdr,
                                                           float* __restrict__ cs) {
  const int t = blockIdx.x, part = blockIdx.y, parts = gridDim.y;
  const int cnt = hdr[kHdrCnt + t];
  if (cnt == 0) return;
  const int off = hdr[kHdrOff + t];
  const int per = (cnt + parts - 1) / parts;
  const int i0 = part * per, i1 = min(cnt, i0 + per);
  for (int f = threadIdx.x; f < H1; f += 256) {
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int i = i0;
    for (; i + 4 <= i1; i += 4) {
      a0 += g1[(size_t)rows[off + i] * H1 + f];
      a1 += g1[(size_t)rows[off + i + 1] * H1 + f];
      a2 += g1[(size_t)rows[off + i + 2] * H1 + f];
      a3 += g1[(size_t)rows[off + i + 3] * H1 + f];
    }
    for (; i < i1; ++i) a0 += g1[(size_t)rows[off + i] * H1 + f];
    if (i0 < i1) atomicAdd(&cs[(size_t)t * H1 + f], (a0 + a1) + (a2 + a3));
  }
}

__global__ __launch_bounds__(256) void bitseq_empty_rows_kernel(const float* __restrict__ cs, int H1, int L, int T,
                                                                int tokens, float* __restrict__ dW1,
                                                                float* __restrict__ db1) {
  const int s = blockIdx.x;  // position
  for (int f = threadIdx.x; f < H1; f += 256) {
    float acc = 0.f;
    for (int t = 0; t <= s && t < T; ++t) acc += cs[(size_t)t * H1 + f];
    dW1[((size_t)(tokens + 1) * s + tokens) * H1 + f] = acc;
    if (s == 0) {
      float tot = 0.f;
      for (int t = 0; t < T; ++t) tot += cs[(size_t)t * H1 + f];
      db1[f] = tot;
    }
  }
  (void)L;
}

// Non-autoregressive bit sequences: the "empty" row of a position is active up to the step that fills it and the row of
// the word written there afterwards, so over the steps of one trajectory the two together are active exactly once per
// step: dW1[empty(s)] = (sum of G1 over all live rows) - sum over the words w of dW1[token(s, w)].  The token rows come
// from the per-trajectory suffix sums (dw1_kernel<3>, suffix_only), the total from the per-step column sums; on average
// the empty row holds half of the total, so the difference loses no accuracy that matters.  The blocks of position 0
// also write db1.
__global__ __launch_bounds__(256) void na_empty_rows_kernel(const float* __restrict__ cs, int H1, int T, int tokens,
                                                            float* __restrict__ dW1, float* __restrict__ db1) {
  // grid (positions, ceil(H1 / 64)): 64 features x four quarters of the word range per block
  __shared__ float red[4][64];
  const int s = blockIdx.x, f = 64 * blockIdx.y + (threadIdx.x & 63), part = threadIdx.x >> 6;
  float a = 0.f;
  if (f < H1) {
    const float* tok = dW1 + (size_t)(tokens + 1) * s * H1 + f;
    for (int w = part; w < tokens; w += 4) a += tok[(size_t)w * H1];
  }
  red[part][threadIdx.x & 63] = a;
  __syncthreads();
  if (part == 0 && f < H1) {
    float tot = 0.f;
    for (int t = 0; t < T; ++t) tot += cs[(size_t)t * H1 + f];
    const int l = threadIdx.x;
    dW1[((size_t)(tokens + 1) * s + tokens) * H1 + f] = tot - ((red[0][l] + red[1][l]) + (red[2][l] + red[3][l]));
    if (s == 0) db1[f] = tot;
  }
}

}  // namespace gfnx

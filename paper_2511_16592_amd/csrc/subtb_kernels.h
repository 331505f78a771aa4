// Subtrajectory Balance / Detailed Balance (Background, eq. SubTB_loss and eq. DB_loss) for a network whose last
// output is log F(s).  With phi_t = log F(s_t) (phi_n = log R), c_t = sum_{i<=t} (log P_F - log P_B) of the first t
// transitions and u_t = phi_t - c_t, the residual of the pair j < k is u_j - u_k, so
//   L(tau) = (1/W) sum_{j<k} lambda^(k-j-1) (u_j - u_k)^2,  W = sum_{j<k} lambda^(k-j-1),
//   g_t = dL/du_t = (2/W) sum_{i != t} lambda^(|i-t|-1) (u_t - u_i),
// log F(s_t) receives g_t and the log-probability of transition t -> t+1 receives -sum_{k>t} g_k.
// lambda = 0 keeps the single-transition pairs only: Detailed Balance averaged over the transitions.
#pragma once
#include "gfnx_device.h"

namespace gfnx {

constexpr int kSubtbMaxSteps = 256;

// One wavefront per trajectory.  In: phi[t*B+b], dl[t*B+b] (log P_F - log P_B of transition t), logr[b].
// Out, in place: phi[t*B+b] = g_t / B, dl[t*B+b] = kappa_t / B (coefficient of d log P_F of transition t),
// lossb[b] = L(tau_b).
__global__ __launch_bounds__(256) void subtb_coef_kernel(const int* __restrict__ length, const float* __restrict__ logr,
                                                         float* __restrict__ phi, float* __restrict__ dl, int B, int T,
                                                         float lambda, float* __restrict__ lossb) {
  __shared__ float us[4][kSubtbMaxSteps + 1], gs[4][kSubtbMaxSteps + 1];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int b = blockIdx.x * 4 + wv;
  if (b >= B) return;  // whole wavefronts leave together; the LDS rows are private to a wavefront
  float* u = us[wv];
  float* g = gs[wv];
  int n = length[b];
  n = n < 1 ? 1 : (n > T ? T : n);
  for (int t = lane; t < n; t += 64) {
    u[t] = phi[(size_t)t * B + b];
    g[t] = dl[(size_t)t * B + b];
  }
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) {  // c_t in the order of the steps, as a sequential sum
    float c = 0.f;
    for (int t = 0; t < n; ++t) {
      const float d = g[t];
      u[t] -= c;
      c += d;
    }
    u[n] = logr[b] - c;
  }
  __builtin_amdgcn_wave_barrier();
  float W = 0.f;  // sum over the distances d = 1..n of (n + 1 - d) lambda^(d-1)
  {
    float w = 1.f;
    for (int d = 1; d <= n; ++d) { W += (float)(n + 1 - d) * w; w *= lambda; }
  }
  const float inv_w = 1.f / W;
  float loss = 0.f;
  for (int t = lane; t <= n; t += 64) {
    const float ut = u[t];
    float acc = 0.f, sq = 0.f, w = 1.f;
    for (int i = t + 1; i <= n; ++i) { const float d = ut - u[i]; acc += w * d; sq += w * d * d; w *= lambda; }
    w = 1.f;
    for (int i = t - 1; i >= 0; --i) { const float d = ut - u[i]; acc += w * d; w *= lambda; }
    g[t] = 2.f * inv_w * acc;
    loss += inv_w * sq;  // every pair once: counted at its smaller index
  }
  for (int o = 32; o > 0; o >>= 1) loss += __shfl_xor(loss, o);
  __builtin_amdgcn_wave_barrier();
  const float inv_b = 1.f / (float)B;
  for (int t = lane; t < n; t += 64) {
    float kappa = 0.f;
    for (int k = t + 1; k <= n; ++k) kappa -= g[k];
    phi[(size_t)t * B + b] = g[t] * inv_b;
    dl[(size_t)t * B + b] = kappa * inv_b;
  }
  if (lane == 0) lossb[b] = loss;
}

// Folds the coefficients into the logit-gradient rows: E[row][a] = kappa[row] E[row][a] for the actions, g[row] for
// the flow output, 0 for the padding; the row coefficient the following kernels multiply by becomes 1.  Block 0
// also sums the per-trajectory losses into the mean (fixed order: strided partial sums, then a tree).
__global__ __launch_bounds__(256) void subtb_apply_kernel(const int* __restrict__ rows, const int* __restrict__ hdr,
                                                          const float* __restrict__ kappa, const float* __restrict__ gflow,
                                                          int n_actions, int A16, float* __restrict__ ebuf,
                                                          float* __restrict__ crow, const float* __restrict__ lossb, int B,
                                                          float* __restrict__ loss) {
  const int n = hdr[kHdrNLive];
  const int cpr = A16 >> 2;  // chunks of four outputs per row
  const size_t total = (size_t)n * cpr;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int pos = (int)(i / cpr), c = (int)(i % cpr);
    const int row = rows[pos];
    const float k = kappa[row], gf = gflow[row];
    f32x4* ep = (f32x4*)&ebuf[(size_t)row * A16 + 4 * c];
    f32x4 v = *ep;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int a = 4 * c + q;
      v[q] = a < n_actions ? k * v[q] : (a == n_actions ? gf : 0.f);
    }
    *ep = v;
    if (c == 0) crow[pos] = 1.f;
  }
  if (blockIdx.x == 0) {  // block-uniform branch
    __shared__ float red[256];
    float acc = 0.f;
    for (int b = threadIdx.x; b < B; b += 256) acc += lossb[b];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) *loss = red[0] / (float)B;
  }
}

}  // namespace gfnx

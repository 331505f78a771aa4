// Backward rollouts and the Monte-Carlo estimate of P_theta(x).
//
// A backward rollout ("Library Details": a rollout started at terminal states with the backward step in place of
// the step; backward actions are the structural choices only) under the fixed uniform backward policy draws, for
// every trajectory, parents of the current state until s_0 is reached.  No network is involved: one lane per
// trajectory, the set of undoable indices (grid: coordinates > 0, Ising: assigned sites, non-autoregressive bit
// sequences: filled positions) as a 128-bit mask in
// registers, the grid's coordinates in LDS.  The j-th undoable index in increasing order is taken, with
// j = floor(w * n / 2^32), w = word 0 of Philox4x32-10(counter = (b, k, 0xFFFFFFFF, iteration lo)), k = index of
// the backward move; the grid's un-stop move and every move of the left-to-right bit sequences have one parent and
// draw nothing.  The trajectory is written in FORWARD order, ready for the teacher-forced rollout that evaluates
// P_F along it.  Then (Appendix "Bit sequences", estimator equation)
//   log P_theta(x) ~= log( (1/N) sum_i P_F(tau^i) / P_B(tau^i | x) ),  tau^i ~ P_B(. | x).
#pragma once
#include "gfnx_device.h"

namespace gfnx {

struct BackwardParams {
  EnvParams env;
  uint32_t seed_lo, seed_hi, iter_lo;
  int B, T;
  const int8_t* term;  // [state_dim][B] terminal states (input)
  uint8_t* actions;    // [T][B]
  uint16_t* actions16; // [T][B], used instead when not null (environments with more than 256 actions)
  int* length;
  float* lpb;
};

constexpr int kBackwardThreads = 64;

__global__ __launch_bounds__(kBackwardThreads) void backward_rollout_kernel(BackwardParams p) {
  __shared__ int8_t coord[16][kBackwardThreads];  // grid coordinates of this lane's state
  __shared__ float neg_log[129];                  // -log n for the number of parents n
  const int lane = threadIdx.x;
  for (int n = 1 + lane; n <= 128; n += kBackwardThreads) neg_log[n] = -logf((float)n);
  __syncthreads();
  const int b = blockIdx.x * kBackwardThreads + lane;
  if (b >= p.B) return;  // no barrier below: every lane works on its own column
  const EnvParams& e = p.env;
  const size_t B = (size_t)p.B;
  int len;
  if (e.kind == 1) {
    // one parent per state: the path is the token sequence itself
    len = e.L;
    const int tok_mask = (1 << e.k_bits) - 1;
    for (int t = 0; t < len; ++t) p.actions[t * B + b] = (uint8_t)(p.term[t * B + b] & tok_mask);
    for (int t = len; t < p.T; ++t) p.actions[t * B + b] = 0xFF;
    p.length[b] = len;
    p.lpb[b] = 0.f;
    return;
  }
  uint32_t m0 = 0, m1 = 0, m2 = 0, m3 = 0;  // undoable indices
  uint32_t s0 = 0, s1 = 0, s2 = 0, s3 = 0;  // Ising: spin +1 at the index
  int moves = 0;
  for (int i = 0; i < e.state_dim; ++i) {
    int v = p.term[i * B + b];
    bool on, up = false;
    if (e.kind == 0) {
      v = v < 0 ? 0 : (v > e.H - 1 ? e.H - 1 : v);  // out-of-range input is clamped into the grid
      coord[i][lane] = (int8_t)v;
      on = v > 0;
      moves += v;
    } else {
      on = true;  // a terminal Ising state has every site assigned (anything not positive counts as -1), a
                  // terminal string of the non-autoregressive bit sequences every position filled
      up = v > 0;
      moves += 1;
    }
    const uint32_t bit = 1u << (i & 31);
    const int q = i >> 5;
    if (on) { m0 |= q == 0 ? bit : 0; m1 |= q == 1 ? bit : 0; m2 |= q == 2 ? bit : 0; m3 |= q == 3 ? bit : 0; }
    if (up) { s0 |= q == 0 ? bit : 0; s1 |= q == 1 ? bit : 0; s2 |= q == 2 ? bit : 0; s3 |= q == 3 ? bit : 0; }
  }
  len = e.kind == 0 ? moves + 1 : moves;
  if (e.kind == 0) p.actions[(size_t)(len - 1) * B + b] = (uint8_t)e.d;  // un-stop: the terminal copy's only parent
  float lpb = 0.f;
  for (int k = 0; k < moves; ++k) {
    const int c0 = __popc(m0), c1 = __popc(m1), c2 = __popc(m2), c3 = __popc(m3);
    const int n = c0 + c1 + c2 + c3;
    uint32_t r[4];
    philox4x32_10((uint32_t)b, (uint32_t)k, 0xFFFFFFFFu, p.iter_lo, p.seed_lo, p.seed_hi, r);
    int j = (int)__umulhi(r[0], (uint32_t)n);
    int q = 0;
    if (j >= c0) { j -= c0; q = 1; if (j >= c1) { j -= c1; q = 2; if (j >= c2) { j -= c2; q = 3; } } }
    uint32_t word = q == 0 ? m0 : q == 1 ? m1 : q == 2 ? m2 : m3;
    int bitpos = 0;  // position of the j-th set bit of the word: halve the range five times
    int c = __popc(word & 0xFFFFu); if (j >= c) { j -= c; bitpos += 16; word >>= 16; }
    c = __popc(word & 0xFFu); if (j >= c) { j -= c; bitpos += 8; word >>= 8; }
    c = __popc(word & 0xFu); if (j >= c) { j -= c; bitpos += 4; word >>= 4; }
    c = __popc(word & 0x3u); if (j >= c) { j -= c; bitpos += 2; word >>= 2; }
    if (j >= (int)(word & 1u)) bitpos += 1;
    const uint32_t bit = 1u << bitpos;
    const int idx = 32 * q + bitpos;
    lpb += neg_log[n];
    int a;
    bool clear;
    if (e.kind == 0) {
      a = idx;
      const int v = coord[idx][lane] - 1;
      coord[idx][lane] = (int8_t)v;
      clear = v == 0;
    } else if (e.kind == 3) {
      // non-autoregressive bit sequences: the word of the position that is emptied
      a = (idx << e.k_bits) + ((int)p.term[(size_t)idx * B + b] & ((1 << e.k_bits) - 1));
      clear = true;
    } else {
      const uint32_t sw = q == 0 ? s0 : q == 1 ? s1 : q == 2 ? s2 : s3;
      a = 2 * idx + ((sw & bit) ? 1 : 0);
      clear = true;
    }
    if (clear) { m0 &= q == 0 ? ~bit : ~0u; m1 &= q == 1 ? ~bit : ~0u; m2 &= q == 2 ? ~bit : ~0u; m3 &= q == 3 ? ~bit : ~0u; }
    // the k-th undone move is forward step moves-1-k
    if (p.actions16) p.actions16[(size_t)(moves - 1 - k) * B + b] = (uint16_t)a;
    else p.actions[(size_t)(moves - 1 - k) * B + b] = (uint8_t)a;
  }
  for (int t = len; t < p.T; ++t) {
    if (p.actions16) p.actions16[t * B + b] = 0xFFFF;
    else p.actions[t * B + b] = 0xFF;
  }
  p.length[b] = len;
  p.lpb[b] = lpb;
}

// One wavefront per state: out[x] = log mean_i exp(log_pf[x*N+i] - log_pb[x*N+i]), shifted by the maximum.
__global__ __launch_bounds__(256) void log_prob_estimate_kernel(const float* __restrict__ lpf, const float* __restrict__ lpb,
                                                                int n_states, int n_samples, float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int x = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (x >= n_states) return;  // whole wavefronts leave together
  const float* f = lpf + (size_t)x * n_samples;
  const float* g = lpb + (size_t)x * n_samples;
  float mx = -INFINITY;
  for (int i = lane; i < n_samples; i += 64) mx = fmaxf(mx, f[i] - g[i]);
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  float acc = 0.f;
  for (int i = lane; i < n_samples; i += 64) acc += expf((f[i] - g[i]) - mx);
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (lane == 0) out[x] = mx + logf(acc / (float)n_samples);
}

}  // namespace gfnx

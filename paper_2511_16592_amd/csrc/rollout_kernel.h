// Persistent trajectory-block rollout kernel.
//
// One workgroup (8 wavefronts, two per SIMD) runs kSlots = 16 trajectories at a time from s_0 to their
// terminal states; it owns a contiguous range of p.tpw trajectories and a slot whose trajectory has ended
// starts the next one of the range (trajectory b is a pure function of (seed, iteration, b), so which slot
// runs it changes nothing).  Per step:
//   L2  hidden layer 2 on the matrix cores, computed transposed: D[feature][slot] = W2^T * relu(z1); the
//       eight waves split the output features; weights are MFMA A-operands (resident in registers when the
//       layer is 256 x 256: 128 registers per lane, or streamed from L2 cache in operand order with the next
//       step's loads in flight), activations come from LDS in B-operand order;
//   L3  logits the same way: output tiles split over the waves, and the contraction split as well when there
//       are fewer than eight tiles;
//   SU  per slot, 32 lanes of one wave: action mask, softmax weights, Philox draw and argmin by DPP row
//       rotations plus one swizzle, log P_F / log P_B, the row of the logit gradient, environment
//       transition, terminal log-reward, action byte; then the same lanes update the layer-1
//       pre-activation: layer 1 is a one-hot gather and a transition swaps exactly one active row, so z1 is
//       kept in LDS (as a high + low pair) and updated as z1 += W1[new] - W1[old].
// The post-ReLU activations h1, h2, their sign masks (1 bit per unit), the state bytes and the logit-gradient
// direction (onehot(a) - p) of every transition are written to HBM rows t*B + b for the gradient pass.  Nothing the
// kernel writes to global memory is read back by it, so the three barriers per step order LDS traffic only
// (no wait for stores to land).
#pragma once
#include "gfnx_device.h"

namespace gfnx {

constexpr int kRolloutWaves = 8;
constexpr int kRolloutThreads = 64 * kRolloutWaves;

template <int ENV>
__device__ __forceinline__ int initial_row(const EnvParams& e, int s) {
  if (ENV == 0) return e.H * s;
  if (ENV == 1) return ((1 << e.k_bits) + 1) * s + (1 << e.k_bits);
  return 3 * s + 1;
}

// k-bit chunk `pos` of packed mode string m (string bit i sits in bit i%32 of word i/32)
__device__ __forceinline__ uint32_t mode_chunk(const uint32_t* modes, int words, int m, int pos, int k) {
  const int s = k * pos;
  const int wd = s >> 5;
  uint64_t v = modes[(size_t)m * words + wd];
  if (wd + 1 < words) v |= (uint64_t)modes[(size_t)m * words + wd + 1] << 32;
  return (uint32_t)(v >> (s & 31)) & ((1u << k) - 1u);
}

__device__ __forceinline__ f32x4 relu4(f32x4 v) {
  v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
  return v;
}

// Sign mask of 256 activations held four per lane (lane l: features 4l .. 4l+3): word k (k < 4) gets bit l
// set iff feature 4l+k is positive.  This is the ReLU derivative the gradient pass needs, at 1 bit per unit.
__device__ __forceinline__ void store_sign_mask(unsigned long long* dst, f32x4 v, int lane) {
  const unsigned long long m0 = __ballot(v.x > 0.f), m1 = __ballot(v.y > 0.f);
  const unsigned long long m2 = __ballot(v.z > 0.f), m3 = __ballot(v.w > 0.f);
  if (lane < 4) dst[lane] = lane == 0 ? m0 : (lane == 1 ? m1 : (lane == 2 ? m2 : m3));
}

// How the logits GEMM is split over the eight waves: with at least eight 16-logit tiles each wave takes
// whole tiles; otherwise the contraction is cut into KS parts so that (tiles x KS) fills the waves.
__host__ __device__ inline int logits_ksplit(int nt3, int q2) {
  if (nt3 >= 8) return 1;
  int ks = 1;
  while (ks * 2 * nt3 <= 8 && q2 % (ks * 2) == 0) ks *= 2;
  return ks;
}

#define GFNX_MFMA4(ACC, AV, BV)            \
  ACC = mfma16((AV).x, (BV).x, ACC);       \
  ACC = mfma16((AV).y, (BV).y, ACC);       \
  ACC = mfma16((AV).z, (BV).z, ACC);       \
  ACC = mfma16((AV).w, (BV).w, ACC)

// NTW  = 16-feature tiles of layer 2 per wave, ceil(H2 / 128).
// STAT = layer 2 is 256 x 256: each wave keeps its two tiles of W2 (32 KiB, 128 registers per lane) in
//        registers for the whole rollout; with a single logit tile (grids) its eighth of W3 as well.
// NCH  = chunks of four logits a lane may own in SU: 1 up to 128 actions, else 2.
template <int ENV, bool REPLAY, int NTW, bool STAT, int NCH>
__global__ __launch_bounds__(kRolloutThreads) void rollout_kernel(const RolloutParams p) {
  extern __shared__ float smem[];
  const EnvParams& e = p.env;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g = lane >> 4, j16 = lane & 15;
  const int H1 = p.H1, H2 = p.H2, A = p.A, A16 = p.A16, B = p.B;
  const int Q1 = H1 >> 4, Q2 = H2 >> 4;
  const int NT2 = H2 >> 4, NT3 = A16 >> 4, nchunk = A16 >> 2;
  const int KS = logits_ksplit(NT3, Q2);

  float* z1s = smem;                          // pre-activation of layer 1, high part
  float* z1l = z1s + (H1 >> 2) * kPitch;      // ... low part (z1 = hi + lo carries the sum to ~48 bits)
  float* h2s = z1l + (H1 >> 2) * kPitch;
  float* lgs = h2s + (H2 >> 2) * kPitch;      // [KS][nchunk] partial logits
  float* z1i = lgs + KS * nchunk * kPitch;    // z1(s_0): [2][H1] high and low parts, for slots that restart
  int* alive = (int*)(z1i + 2 * H1);          // [kSlots] slot is running a trajectory
  int* srow = alive + kSlots;                 // [kSlots] row t*B + b of the slot's current transition
  int* qnext = srow + kSlots;                 // next trajectory of this workgroup's range to start
  int8_t* st = (int8_t*)(qnext + 4);

  const int b0 = blockIdx.x * p.tpw;                    // this workgroup's trajectories: [b0, bend)
  const int bend = min(B, b0 + p.tpw);
  // roles in the SU phase: 32 lanes (sub-lane si) of one wave per slot sj
  const int sj = 2 * w + (lane >> 5), si = lane & 31;
  int sb = b0 + sj;                                     // trajectory in this slot
  int ts = 0;                                           // its step counter

  // ---- reset: s_0, z1(s_0) = b1 + sum of the initially active rows
  for (int f = tid; f < H1; f += kRolloutThreads) {
    double z = (double)p.b1[f];
    for (int s = 0; s < e.state_dim; ++s) z += (double)p.W1[(size_t)initial_row<ENV>(e, s) * H1 + f];
    const float hi = (float)z, lo = (float)(z - (double)hi);
    float* dh = z1s + (f >> 2) * kPitch + (f & 3);
    float* dl = z1l + (f >> 2) * kPitch + (f & 3);
#pragma unroll
    for (int j = 0; j < kSlots; ++j) { dh[j * 4] = hi; dl[j * 4] = lo; }
    z1i[f] = hi;
    z1i[H1 + f] = lo;
  }
  for (int i = tid; i < e.state_dim * kSlots; i += kRolloutThreads) st[i] = 0;
  if (tid < kSlots) {
    alive[tid] = (b0 + tid < bend) ? 1 : 0;
    srow[tid] = b0 + tid;
  }
  if (tid == 0) *qnext = b0 + kSlots;
  float lpf = 0.f, lpb = 0.f;
  int len_given = 0;
  if (REPLAY && sb < bend) len_given = p.length[sb];
  f32x4 w2r[STAT ? 2 : 1][STAT ? 16 : 1];
  f32x4 w3r[STAT ? 2 : 1];
  if constexpr (STAT) {
    const f32x4* wp = (const f32x4*)p.W2p + (size_t)(w * 2) * 16 * 64 + lane;
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int q = 0; q < 16; ++q) w2r[n][q] = wp[(n * 16 + q) * 64];
    const f32x4* wp3 = (const f32x4*)p.W3p + lane;  // tile 0, this wave's eighth of the contraction
#pragma unroll
    for (int q = 0; q < 2; ++q) w3r[q] = wp3[(w * 2 + q) * 64];
  }
  lds_barrier();

  // list-scheduling bound on the number of steps: (sum of lengths) / kSlots + longest trajectory
  const int max_iters = e.max_steps * ((p.tpw + kSlots - 1) / kSlots + 1);
  for (int iter = 0; iter < max_iters; ++iter) {
    // ================= L2: h2 = relu(W2^T relu(z1) + b2)
    for (int jj = w; jj < kSlots; jj += kRolloutWaves) {
      if (!alive[jj]) continue;
      const size_t row = (size_t)srow[jj];
      float* dst = p.h1buf + row * H1;
      for (int it = 0; it * 64 < (H1 >> 2); ++it) {
        const int fg = lane + 64 * it;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (fg < (H1 >> 2)) {
          v = relu4(*(const f32x4*)&z1s[fg * kPitch + jj * 4]);
          *(f32x4*)&dst[fg * 4] = v;
        }
        store_sign_mask(p.m1buf + (row * p.MW1 + 4 * it), v, lane);
      }
    }
    {
      f32x4 acc[NTW];
#pragma unroll
      for (int n = 0; n < NTW; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if constexpr (STAT) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const f32x4 bv = relu4(*(const f32x4*)&z1s[(4 * q + g) * kPitch + j16 * 4]);
#pragma unroll
          for (int n = 0; n < 2; ++n) { GFNX_MFMA4(acc[n], w2r[n][q], bv); }
        }
      } else if (w * NTW < NT2) {
        // tiles w*NTW .. w*NTW+NTW-1 (clamped: a clamped tile is computed twice and stored once)
        const f32x4* wp = (const f32x4*)p.W2p + lane;
        int tn[NTW];
#pragma unroll
        for (int n = 0; n < NTW; ++n) tn[n] = min(w * NTW + n, NT2 - 1);
        f32x4 cur[NTW];
#pragma unroll
        for (int n = 0; n < NTW; ++n) cur[n] = wp[((size_t)tn[n] * Q1) * 64];
        for (int q = 0; q < Q1; ++q) {
          const int qn = q + 1 < Q1 ? q + 1 : q;
          f32x4 nxt[NTW];
#pragma unroll
          for (int n = 0; n < NTW; ++n) nxt[n] = wp[((size_t)tn[n] * Q1 + qn) * 64];
          const f32x4 bv = relu4(*(const f32x4*)&z1s[(4 * q + g) * kPitch + j16 * 4]);
#pragma unroll
          for (int n = 0; n < NTW; ++n) { GFNX_MFMA4(acc[n], cur[n], bv); }
#pragma unroll
          for (int n = 0; n < NTW; ++n) cur[n] = nxt[n];
        }
      }
#pragma unroll
      for (int n = 0; n < NTW; ++n) {
        const int nt = w * NTW + n;
        if (nt < NT2) {
          const f32x4 bias = *(const f32x4*)&p.b2[16 * nt + 4 * g];
          *(f32x4*)&h2s[(4 * nt + g) * kPitch + j16 * 4] = relu4(acc[n] + bias);
        }
      }
    }
    lds_barrier();

    // ================= L3: logits = W3^T h2 (+ b3 added in SU)
    for (int jj = w; jj < kSlots; jj += kRolloutWaves) {
      if (!alive[jj]) continue;
      const size_t row = (size_t)srow[jj];
      float* dst = p.h2buf + row * H2;
      for (int it = 0; it * 64 < (H2 >> 2); ++it) {
        const int fg = lane + 64 * it;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (fg < (H2 >> 2)) {
          v = *(const f32x4*)&h2s[fg * kPitch + jj * 4];
          *(f32x4*)&dst[fg * 4] = v;
        }
        store_sign_mask(p.m2buf + (row * p.MW2 + 4 * it), v, lane);
      }
    }
    if (KS == 1) {
      // whole tiles: w and w + 8
      f32x4 acc[2];
#pragma unroll
      for (int n = 0; n < 2; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (w < NT3) {
        const f32x4* wp = (const f32x4*)p.W3p + lane;
        const int t0 = w, t1 = min(w + 8, NT3 - 1);
        f32x4 c0 = wp[((size_t)t0 * Q2) * 64], c1 = wp[((size_t)t1 * Q2) * 64];
        for (int q = 0; q < Q2; ++q) {
          const int qn = q + 1 < Q2 ? q + 1 : q;
          const f32x4 n0 = wp[((size_t)t0 * Q2 + qn) * 64], n1 = wp[((size_t)t1 * Q2 + qn) * 64];
          const f32x4 bv = *(const f32x4*)&h2s[(4 * q + g) * kPitch + j16 * 4];
          GFNX_MFMA4(acc[0], c0, bv);
          if (w + 8 < NT3) { GFNX_MFMA4(acc[1], c1, bv); }
          c0 = n0; c1 = n1;
        }
        *(f32x4*)&lgs[(4 * w + g) * kPitch + j16 * 4] = acc[0];
        if (w + 8 < NT3) *(f32x4*)&lgs[(4 * (w + 8) + g) * kPitch + j16 * 4] = acc[1];
      }
    } else {
      // wave w: tile w / KS, contraction part w % KS
      const int nt = w / KS, ks = w - nt * KS;
      if (nt < NT3) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        const int qn = Q2 / KS;
        if (STAT && NT3 == 1 && KS == 8) {
#pragma unroll
          for (int q = 0; q < (STAT ? 2 : 1); ++q) {
            const f32x4 bv = *(const f32x4*)&h2s[(4 * (w * 2 + q) + g) * kPitch + j16 * 4];
            GFNX_MFMA4(acc, w3r[q], bv);
          }
        } else {
          const f32x4* wp = (const f32x4*)p.W3p + lane;
          for (int q = ks * qn; q < (ks + 1) * qn; ++q) {
            const f32x4 bv = *(const f32x4*)&h2s[(4 * q + g) * kPitch + j16 * 4];
            const f32x4 av = wp[((size_t)nt * Q2 + q) * 64];
            GFNX_MFMA4(acc, av, bv);
          }
        }
        *(f32x4*)&lgs[(ks * nchunk + 4 * nt + g) * kPitch + j16 * 4] = acc;
      }
    }
    lds_barrier();

    // ================= SU: mask, softmax, sample, bookkeeping, transition, z1 update (32 lanes per slot)
    if (alive[sj]) {
      const int t = ts;
      if (p.sbuf) {  // the state the policy is evaluated at, for the one-hot contraction of the gradient pass
        uint32_t* srowp = (uint32_t*)(p.sbuf + ((size_t)t * B + sb) * p.SB);  // SB is a multiple of 16
        for (int s4 = si; 4 * s4 < p.SB; s4 += 32) {
          uint32_t packed = 0;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int s = 4 * s4 + k;
            const uint32_t byte = s < e.state_dim ? (uint32_t)(uint8_t)st[s * kSlots + sj] : 0u;
            packed |= byte << (8 * k);
          }
          srowp[s4] = packed;
        }
      }
      f32x4 lg[NCH];
      uint32_t vm[NCH];
      float m = -INFINITY;
#pragma unroll
      for (int n = 0; n < NCH; ++n) {
        const int c = si + 32 * n;
        vm[n] = 0;
        lg[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (c < nchunk) {
          f32x4 v;
#pragma unroll
          for (int k = 0; k < 4; ++k) v[k] = (4 * c + k < A) ? p.b3[4 * c + k] : 0.f;
          for (int ks = 0; ks < KS; ++ks) v += *(const f32x4*)&lgs[(ks * nchunk + c) * kPitch + sj * 4];
          lg[n] = v;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            // branch-free: state bytes are read at a clamped index and combined with bitwise logic
            const int a = 4 * c + k;
            uint32_t ok;
            if (ENV == 0) {
              const int sv = st[min(a, e.d - 1) * kSlots + sj];
              ok = (uint32_t)(a == e.d) | ((uint32_t)(a < e.d) & (uint32_t)(sv < e.H - 1));
            } else if (ENV == 1) {
              ok = (uint32_t)(a < A);
            } else {
              const int sv = st[min(a >> 1, e.D - 1) * kSlots + sj];
              ok = (uint32_t)(a < A) & (uint32_t)(sv == 0);
            }
            vm[n] |= ok << k;
            m = ok ? fmaxf(m, v[k]) : m;
          }
        }
      }
      m = grp32_max(m);
      // softmax weights exp(l - m) of the valid actions (0 elsewhere) and their sum
      f32x4 wv[NCH];
      float sum = 0.f;
#pragma unroll
      for (int n = 0; n < NCH; ++n)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          wv[n][k] = ((vm[n] >> k) & 1u) ? expf(lg[n][k] - m) : 0.f;
          sum += wv[n][k];
        }
      sum = grp32_sum(sum);
      const float lse = logf(sum);
      const float inv_sum = 1.f / sum;

      int act;
      float alogit;
      bool given_ok = true;  // teacher-forced mode: is the given action possible in this state?
      if (!REPLAY) {
        // Gumbel-max as an exponential race: argmax_a (l_a - log(-log u_a)) = argmin_a (-log u_a) / exp(l_a - m),
        // one logarithm per action; lowest index wins exact ties
        float best = INFINITY, blog = 0.f;
        int bidx = 0x7fffffff;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
          const int c = si + 32 * n;
          if (vm[n]) {
            uint32_t wd[4];
            philox4x32_10((uint32_t)sb, (uint32_t)t, (uint32_t)c, p.iter_lo, p.seed_lo, p.seed_hi, wd);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              if ((vm[n] >> k) & 1u) {
                const float r = -logf(uniform_from_bits(wd[k])) / wv[n][k];
                if (r < best) { best = r; bidx = 4 * c + k; blog = lg[n][k]; }
              }
            }
          }
        }
        grp32_argmin(best, bidx, blog);
        act = bidx;
        alogit = blog;
      } else {
        act = p.actions[(size_t)t * B + sb];
        float mine = 0.f;
        int mine_ok = 0;
#pragma unroll
        for (int n = 0; n < NCH; ++n)
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (4 * (si + 32 * n) + k == act) { mine = lg[n][k]; mine_ok = (int)((vm[n] >> k) & 1u); }
        alogit = __shfl(mine, (act >> 2) & 31, 32);
        given_ok = __shfl(mine_ok, (act >> 2) & 31, 32) != 0;
        if (!given_ok) { act = 0; alogit = m + lse; }  // log p = 0; the trajectory is cut below
      }
      lpf += (alogit - m) - lse;

      {  // direction of the logit gradient: onehot(a) - p on valid actions, 0 elsewhere
        float* erow = p.ebuf + ((size_t)t * B + sb) * A16;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
          const int c = si + 32 * n;
          if (c < nchunk) {
            f32x4 ev;
#pragma unroll
            for (int k = 0; k < 4; ++k)
              ev[k] = ((vm[n] >> k) & 1u) ? ((4 * c + k == act ? 1.f : 0.f) - wv[n][k] * inv_sum) : 0.f;
            *(f32x4*)&erow[4 * c] = ev;
          }
        }
      }

      bool term = false;
      float logr = 0.f;
      int xi = 0;              // grid: this lane's coordinate after the step
      int site = 0, spin = 0;  // ising
      int rold = 0, rnew = 0;  // the one-hot row that leaves / enters (known to all lanes of the slot)
      if (REPLAY && !given_ok) {
        term = true;  // impossible action in the given sequence: cut the trajectory here, state unchanged
        if (ENV == 0) xi = (si < e.d) ? st[si * kSlots + sj] : 0;
        site = -1;
      } else if (ENV == 0) {
        xi = (si < e.d) ? st[si * kSlots + sj] : 0;
        if (act != e.d) {
          const int xa = st[act * kSlots + sj];
          rold = e.H * act + xa;
          rnew = rold + 1;
          if (si == act) { st[si * kSlots + sj] = (int8_t)(xi + 1); xi += 1; }
          const int cnt = grp32_sum((si < e.d && xi > 0) ? 1 : 0);
          lpb -= logf((float)cnt);
        } else {
          const float v = fabsf((float)xi / (float)(e.H - 1) - 0.5f);
          const int bad1 = grp32_sum((si < e.d && !(0.25f < v)) ? 1 : 0);
          const int bad2 = grp32_sum((si < e.d && !((0.3f < v) && (v < 0.4f))) ? 1 : 0);
          const float r = e.r0 + e.r1 * (bad1 == 0 ? 1.f : 0.f) + e.r2 * (bad2 == 0 ? 1.f : 0.f);
          logr = logf(r);
          term = true;
        }
      } else if (ENV == 1) {
        const int k = e.k_bits;
        rold = ((1 << k) + 1) * t + (1 << k);
        rnew = ((1 << k) + 1) * t + act;
        if (si == 0) st[t * kSlots + sj] = (int8_t)act;
        if (t == e.L - 1) {
          int dmin = 0x7fffffff;
          for (int mm = si; mm < e.n_modes; mm += 32) {
            int dist = 0;
            for (int pos = 0; pos < e.L; ++pos) {
              const uint32_t tok = (pos == t) ? (uint32_t)act : (uint32_t)(uint8_t)st[pos * kSlots + sj];
              const uint32_t rev = __brev(tok) >> (32 - k);
              dist += __popc(rev ^ mode_chunk(e.modes, e.words, mm, pos, k));
            }
            dmin = min(dmin, dist);
          }
          dmin = grp32_min(dmin);
          logr = -(e.beta / (float)e.n_bits) * (float)dmin;
          term = true;
        }
      } else {
        site = act >> 1;
        spin = 2 * (act & 1) - 1;
        rold = 3 * site + 1;
        rnew = 3 * site + 1 + spin;
        if (si == 0) st[site * kSlots + sj] = (int8_t)spin;
        lpb -= logf((float)(t + 1));
        if (t == e.D - 1) {
          int acc = 0;
          for (int s = si; s < e.D; s += 32) {
            const int r = s / e.N, c = s - r * e.N;
            const int sr = r * e.N + (c + 1 == e.N ? 0 : c + 1);
            const int sd = (r + 1 == e.N ? 0 : r + 1) * e.N + c;
            const int x = (s == site) ? spin : st[s * kSlots + sj];
            const int xr = (sr == site) ? spin : st[sr * kSlots + sj];
            const int xd = (sd == site) ? spin : st[sd * kSlots + sj];
            acc += x * (xr + xd);
          }
          acc = grp32_sum(acc);
          logr = e.coupling * (float)acc;
          term = true;
        }
      }
      if (REPLAY) term = term || (t + 1 >= len_given);
      if (!REPLAY && si == 0) p.actions[(size_t)t * B + sb] = (uint8_t)act;
      if (term) {
        if (si == 0) {
          if (!REPLAY) p.length[sb] = t + 1;
          p.lpf[sb] = lpf;
          p.lpb[sb] = lpb;
          p.logr[sb] = logr;
        }
        for (int s = si; s < e.state_dim; s += 32) {
          int v;
          if (ENV == 0) v = xi;  // state_dim <= 16: lane s holds coordinate s
          else if (ENV == 1) v = (s == t && given_ok) ? act : (int)(uint8_t)st[s * kSlots + sj];
          else v = (s == site) ? spin : st[s * kSlots + sj];
          p.term[(size_t)s * B + sb] = (int8_t)v;
        }
        // the slot starts the next trajectory of the workgroup's range, if any is left
        int nb = 0;
        if (si == 0) nb = atomicAdd(qnext, 1);
        nb = __shfl(nb, 0, 32);
        if (nb < bend) {
          sb = nb;
          ts = 0;
          lpf = 0.f;
          lpb = 0.f;
          if (REPLAY) len_given = p.length[sb];
          for (int s2 = si; s2 < e.state_dim; s2 += 32) st[s2 * kSlots + sj] = 0;
          for (int fg = si; fg < (H1 >> 2); fg += 32) {
            *(f32x4*)&z1s[fg * kPitch + sj * 4] = *(const f32x4*)&z1i[4 * fg];
            *(f32x4*)&z1l[fg * kPitch + sj * 4] = *(const f32x4*)&z1i[H1 + 4 * fg];
          }
          if (si == 0) srow[sj] = sb;
        } else if (si == 0) {
          alive[sj] = 0;
        }
      } else {
        ts = t + 1;
        if (si == 0) srow[sj] = ts * B + sb;
        // z1 += W1[new row] - W1[old row] for this slot; the running sum is carried as hi + lo so that,
        // however long the walk, relu and its derivative see the correctly rounded sum of the active rows
        const float* wo_row = p.W1 + (size_t)rold * H1;
        const float* wn_row = p.W1 + (size_t)rnew * H1;
        for (int fg = si; fg < (H1 >> 2); fg += 32) {
          f32x4* zp = (f32x4*)&z1s[fg * kPitch + sj * 4];
          f32x4* lp = (f32x4*)&z1l[fg * kPitch + sj * 4];
          const f32x4 wo = *(const f32x4*)&wo_row[4 * fg];
          const f32x4 wn = *(const f32x4*)&wn_row[4 * fg];
          f32x4 hi = *zp, lo = *lp;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const double z = ((double)hi[k] + (double)lo[k]) - (double)wo[k] + (double)wn[k];
            hi[k] = (float)z;
            lo[k] = (float)(z - (double)hi[k]);
          }
          *zp = hi;
          *lp = lo;
        }
      }
    }
    lds_barrier();
    {
      const int4* av = (const int4*)alive;
      const int4 a0 = av[0], a1 = av[1], a2 = av[2], a3 = av[3];
      const int any = a0.x | a0.y | a0.z | a0.w | a1.x | a1.y | a1.z | a1.w | a2.x | a2.y | a2.z | a2.w | a3.x |
                      a3.y | a3.z | a3.w;
      if (!any) break;
    }
  }
}

// W[K][N] row-major -> MFMA A-operand order: out[nt][q][lane][s] = W[16q + 4*(lane/16) + s][16nt + lane%16],
// zero beyond column N.
__global__ void pack_weights_kernel(const float* __restrict__ W, int K, int N, int NT, float* __restrict__ out) {
  const int Q = K >> 4;
  const size_t total = (size_t)NT * Q * 256;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int s = (int)(i & 3), ln = (int)((i >> 2) & 63);
    const size_t r = i >> 8;
    const int q = (int)(r % Q), nt = (int)(r / Q);
    const int k = 16 * q + 4 * (ln >> 4) + s, n = 16 * nt + (ln & 15);
    out[i] = n < N ? W[(size_t)k * N + n] : 0.f;
  }
}

}  // namespace gfnx

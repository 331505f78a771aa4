// Rollout of the non-autoregressive bit sequences (Appendix "Sequential environments", non-autoregressive scheme;
// Appendix "Bit sequences") when the action space is wider than one logit tile of the general kernel: more than 256
// actions, a multiple of 256 (the paper's instance: 15 positions x 256 words = 3840 actions).
//
// One workgroup of 8 waves runs 16 trajectory slots in lockstep (every trajectory has exactly L steps), one group of 16
// trajectories after the other.  Per step:
//   L1   z1 = b1 + sum of the L active rows of W1 (position p contributes the row of its word, or of "empty"), summed
//        in binary64 from scratch, h1 = relu(z1) to LDS (B-operand order) and, with its bit plane, to HBM;
//   L2   h2 = relu(W2^T h1 + b2) on the binary32 matrix cores, W2 streamed from L2 cache in operand order;
//   L3   the logits in pages of 256 actions (16 tiles, two per wave), W3 streamed from L2 cache; after each page the
//        32 lanes of a slot take their 8 logits of the page: mask (position filled?), raw logit (-inf where masked)
//        to HBM for the gradient pass, per-lane running maximum and sum of exp (online softmax), per-lane running
//        Gumbel-max (Philox counter (b, t, a / 4, iteration) as everywhere, key l_a - log(-log u_a): no common
//        maximum is needed across pages).  One barrier per page: the page tile is double-buffered in LDS;
//   SU   the lanes' maxima, sums and best keys meet (DPP / swizzle reductions), log P_F, the row's log-sum-exp to
//        HBM, transition, log P_B -= log(t+1), reward after the last step.
// REPLAY follows given actions instead of sampling (an impossible action cuts the trajectory, as in the general kernel).
// Epsilon-uniform exploration (free-running only): one more Philox call per step, counter (b, t, 0xFFFFFFFE, iteration);
// word 0 decides, word 1 picks the j-th valid action in increasing order -- here simply word j mod 2^k of the
// (j div 2^k)-th empty position, known before the logits are.
#pragma once
#include "gfnx_device.h"
#include "grad_kernels.h"
#include "rollout_kernel.h"

namespace gfnx {

struct WideParams {
  EnvParams env;
  int In, H1, H2, A;  // A = L * 2^k, a multiple of 256
  const float *W1, *b1, *b2, *b3;
  const float *W2p, *W3p;  // weights in MFMA A-operand order (pack_weights_part)
  uint32_t seed_lo, seed_hi, iter_lo;
  int B, T;
  int tpw;  // trajectories owned by one workgroup (a multiple of kSlots)
  uint16_t* actions;  // [T][B]
  int* length;
  int8_t* term;
  float *lpf, *lpb, *logr;
  float *h1buf, *h2buf;  // per-transition rows, row = t*B + b
  float* lgbuf;          // [row][A] logits of the row, -inf where the action is masked
  float* lsebuf;         // [row] log-sum-exp of the valid logits (NaN: the row carries no gradient)
  unsigned long long *m1buf, *m2buf;
  int MW1, MW2;
  float eps;  // epsilon-uniform exploration: probability of a uniform draw over the valid actions (0 = off)
};

struct WideLds {
  int h1s, h2s, lgs, words, filled, total;
};
__host__ __device__ inline WideLds wide_lds_layout(int H1, int H2) {
  WideLds L;
  int o = 0;
  L.h1s = o; o += (H1 >> 2) * kPitch * 4;
  L.h2s = o; o += (H2 >> 2) * kPitch * 4;
  L.lgs = o; o += 2 * 64 * kPitch * 4;  // two page tiles of 256 logits x 16 slots
  L.words = o; o += kSlots * 32;        // word written at each position (L <= 32)
  L.filled = o; o += kSlots * 4;        // bit p: position p is filled
  L.total = o;
  return L;
}

// order-preserving map of a float to an unsigned integer (larger float <-> larger integer)
__device__ __forceinline__ uint32_t float_order(float y) {
  const uint32_t b = __builtin_bit_cast(uint32_t, y);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <bool REPLAY>
__global__ __launch_bounds__(kRolloutThreads) void rollout_wide_kernel(const WideParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const EnvParams& e = p.env;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g = lane >> 4, j16 = lane & 15;
  const int H1 = p.H1, H2 = p.H2, A = p.A, B = p.B;
  const int Q1 = H1 >> 4, Q2 = H2 >> 4, NT2 = H2 >> 4, NP = A >> 8;
  const int kb = e.k_bits, nw = 1 << kb, Lp = e.L;
  constexpr int NTW = 4;  // layer-2 tiles per wave (hidden widths up to 512)

  const WideLds Ld = wide_lds_layout(H1, H2);
  float* h1s = (float*)(smem_raw + Ld.h1s);
  float* h2s = (float*)(smem_raw + Ld.h2s);
  float* lgs = (float*)(smem_raw + Ld.lgs);
  uint8_t* words = smem_raw + Ld.words;
  uint32_t* filled = (uint32_t*)(smem_raw + Ld.filled);

  const int b0 = blockIdx.x * p.tpw, bend = min(B, b0 + p.tpw);
  const int sj = 2 * w + (lane >> 5), si = lane & 31;  // slot and sub-lane of this lane in the per-slot parts

  f32x4 b2r[NTW];
#pragma unroll
  for (int n = 0; n < NTW; ++n) b2r[n] = *(const f32x4*)&p.b2[16 * min(w * NTW + n, NT2 - 1) + 4 * g];

  for (int grp = b0; grp < bend; grp += kSlots) {
    const int sb = grp + sj;              // trajectory of this lane's slot
    bool running = sb < bend;             // (REPLAY: until its given actions end or turn out impossible)
    int len_given = Lp;
    if (REPLAY && running) len_given = min(p.length[sb], Lp);
    if (REPLAY && len_given <= 0) running = false;
    float lpf = 0.f, lpb = 0.f;
    for (int i = tid; i < kSlots * 32 / 4; i += kRolloutThreads) ((uint32_t*)words)[i] = 0u;
    if (tid < kSlots) filled[tid] = 0u;
    lds_barrier();

    for (int t = 0; t < Lp; ++t) {
      // ================= L1: z1 from scratch in binary64; h1 rows and bit planes of slots w and w + 8
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int jj = w + 8 * hh;
        const bool on = grp + jj < bend;
        const size_t row = (size_t)t * B + (size_t)(grp + jj);
        const uint32_t fl = filled[jj];
        for (int it = 0; it * 64 < (H1 >> 2); ++it) {
          const int fg = lane + 64 * it;
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          if (fg < (H1 >> 2)) {
            if (on) {
              const f32x4 bb = *(const f32x4*)&p.b1[4 * fg];
              double z0 = bb.x, z1 = bb.y, z2 = bb.z, z3 = bb.w;
              for (int p0 = 0; p0 < Lp; p0 += 8) {  // eight rows requested together, added in position order
                f32x4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                  const int pos = min(p0 + u, Lp - 1);
                  const int r = (nw + 1) * pos + (((fl >> pos) & 1u) ? (int)words[jj * 32 + pos] : nw);
                  x[u] = *(const f32x4*)&p.W1[(size_t)r * H1 + 4 * fg];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                  if (p0 + u < Lp) {
                    z0 += (double)x[u].x; z1 += (double)x[u].y; z2 += (double)x[u].z; z3 += (double)x[u].w;
                  }
                }
              }
              v = (f32x4){relu1((float)z0), relu1((float)z1), relu1((float)z2), relu1((float)z3)};
              *(f32x4*)&p.h1buf[row * H1 + 4 * fg] = v;
            }
            *(f32x4*)&h1s[fg * kPitch + jj * 4] = v;
          }
          if (on) store_sign_mask(p.m1buf + (row * p.MW1 + 4 * it), v, lane);
        }
      }
      lds_barrier();

      // ================= L2: h2 = relu(W2^T h1 + b2); tiles w*NTW .. w*NTW+NTW-1 (clamped: computed twice, stored once)
      if (w * NTW < NT2) {
        f32x4 acc[NTW];
#pragma unroll
        for (int n = 0; n < NTW; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
        const f32x4* wp = (const f32x4*)p.W2p + lane;
        const f32x4* wt[NTW];
#pragma unroll
        for (int n = 0; n < NTW; ++n) wt[n] = wp + (size_t)min(w * NTW + n, NT2 - 1) * Q1 * 64;
        f32x4 r[2][NTW];
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
          for (int n = 0; n < NTW; ++n) r[d][n] = wt[n][min(d, Q1 - 1) * 64];
        f32x4 bvn = *(const f32x4*)&h1s[g * kPitch + j16 * 4];
#pragma nounroll
        for (int q0 = 0; q0 < Q1; q0 += 2) {  // Q1 is a multiple of 4
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const int q = q0 + d;
            f32x4 cur[NTW];
#pragma unroll
            for (int n = 0; n < NTW; ++n) cur[n] = r[d][n];
            const int qn = min(q + 2, Q1 - 1);
#pragma unroll
            for (int n = 0; n < NTW; ++n) r[d][n] = wt[n][qn * 64];
            const f32x4 bv = bvn;
            bvn = *(const f32x4*)&h1s[(4 * min(q + 1, Q1 - 1) + g) * kPitch + j16 * 4];
#pragma unroll
            for (int n = 0; n < NTW; ++n) acc[n] = mfma16(cur[n].x, bv.x, acc[n]);
#pragma unroll
            for (int n = 0; n < NTW; ++n) acc[n] = mfma16(cur[n].y, bv.y, acc[n]);
#pragma unroll
            for (int n = 0; n < NTW; ++n) acc[n] = mfma16(cur[n].z, bv.z, acc[n]);
#pragma unroll
            for (int n = 0; n < NTW; ++n) acc[n] = mfma16(cur[n].w, bv.w, acc[n]);
            __builtin_amdgcn_sched_group_barrier(0x020, NTW, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * NTW, 0);
          }
        }
#pragma unroll
        for (int n = 0; n < NTW; ++n) {
          const int nt = w * NTW + n;
          if (nt < NT2) *(f32x4*)&h2s[(4 * nt + g) * kPitch + j16 * 4] = relu4(acc[n] + b2r[n]);
        }
      }
      lds_barrier();

      // h2 rows and bit planes of slots w and w + 8
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int jj = w + 8 * hh;
        if (grp + jj >= bend) continue;
        const size_t row = (size_t)t * B + (size_t)(grp + jj);
        for (int it = 0; it * 64 < (H2 >> 2); ++it) {
          const int fg = lane + 64 * it;
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          if (fg < (H2 >> 2)) {
            v = *(const f32x4*)&h2s[fg * kPitch + jj * 4];
            *(f32x4*)&p.h2buf[row * H2 + 4 * fg] = v;
          }
          store_sign_mask(p.m2buf + (row * p.MW2 + 4 * it), v, lane);
        }
      }

      // ================= L3 + per-page part of SU
      const size_t myrow = (size_t)t * B + (size_t)sb;
      const uint32_t myfill = filled[sj];
      int given = -1;  // REPLAY: the action to follow; free-running: the explored action of this step, if any
      if (REPLAY && running) given = p.actions[myrow];
      if (!REPLAY && p.eps > 0.f && running) {
        uint32_t we[4];
        philox4x32_10_ukey((uint32_t)sb, (uint32_t)t, 0xFFFFFFFEu, p.iter_lo, p.seed_lo, p.seed_hi, we);
        if (uniform_from_bits(we[0]) < p.eps) {
          const int j = (int)__umulhi(we[1], (uint32_t)((Lp - t) << kb));  // Lp - t positions are empty
          int left = j >> kb, pos_e = 0;
          for (int q = 0; q < Lp; ++q) {
            const bool empty = ((myfill >> q) & 1u) == 0u;
            if (empty && left == 0) { pos_e = q; break; }
            left -= empty ? 1 : 0;
          }
          given = (pos_e << kb) | (j & (nw - 1));
        }
      }
      float m_run = -INFINITY, s_run = 0.f;  // online softmax of this lane's logits
      unsigned long long best = ~0ull;       // (inverted order of the Gumbel key, action): smallest wins
      float l_best = 0.f;                    // logit of this lane's best (REPLAY: of the given action, if this lane owns it)
      for (int page = 0; page < NP; ++page) {
        float* lgp = lgs + (page & 1) * 64 * kPitch;
        {
          // tiles 16 page + w and 16 page + w + 8: two independent accumulator chains, weights two steps ahead
          constexpr int kL3Ahead = 4;
          f32x4 acc[2];
#pragma unroll
          for (int n = 0; n < 2; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
          const f32x4* wp0 = (const f32x4*)p.W3p + (size_t)(16 * page + w) * Q2 * 64 + lane;
          const f32x4* wp1 = (const f32x4*)p.W3p + (size_t)(16 * page + w + 8) * Q2 * 64 + lane;
          f32x4 r0[kL3Ahead], r1[kL3Ahead];
#pragma unroll
          for (int d = 0; d < kL3Ahead; ++d) {
            r0[d] = wp0[min(d, Q2 - 1) * 64];
            r1[d] = wp1[min(d, Q2 - 1) * 64];
          }
          f32x4 bvn = *(const f32x4*)&h2s[g * kPitch + j16 * 4];
#pragma nounroll
          for (int q0 = 0; q0 < Q2; q0 += kL3Ahead) {
#pragma unroll
            for (int d = 0; d < kL3Ahead; ++d) {
              const int q = q0 + d;
              const f32x4 c0 = r0[d], c1 = r1[d];
              const int qn = min(q + kL3Ahead, Q2 - 1);
              r0[d] = wp0[qn * 64];
              r1[d] = wp1[qn * 64];
              const f32x4 bv = bvn;
              bvn = *(const f32x4*)&h2s[(4 * min(q + 1, Q2 - 1) + g) * kPitch + j16 * 4];
              acc[0] = mfma16(c0.x, bv.x, acc[0]); acc[1] = mfma16(c1.x, bv.x, acc[1]);
              acc[0] = mfma16(c0.y, bv.y, acc[0]); acc[1] = mfma16(c1.y, bv.y, acc[1]);
              acc[0] = mfma16(c0.z, bv.z, acc[0]); acc[1] = mfma16(c1.z, bv.z, acc[1]);
              acc[0] = mfma16(c0.w, bv.w, acc[0]); acc[1] = mfma16(c1.w, bv.w, acc[1]);
              __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
            }
          }
          *(f32x4*)&lgp[(4 * w + g) * kPitch + j16 * 4] = acc[0];
          *(f32x4*)&lgp[(4 * (w + 8) + g) * kPitch + j16 * 4] = acc[1];
        }
        lds_barrier();
        if (running) {
#pragma unroll
          for (int n = 0; n < 2; ++n) {
            const int c = si + 32 * n;       // chunk of four actions within the page
            const int a0 = 256 * page + 4 * c;
            f32x4 lg = *(const f32x4*)&lgp[c * kPitch + sj * 4] + *(const f32x4*)&p.b3[a0];
            uint32_t ok = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) ok |= (((myfill >> ((a0 + k) >> kb)) & 1u) ^ 1u) << k;
            f32x4 out;
#pragma unroll
            for (int k = 0; k < 4; ++k) out[k] = ((ok >> k) & 1u) ? lg[k] : -INFINITY;
            *(f32x4*)&p.lgbuf[myrow * A + a0] = out;
            // online softmax over this lane's valid logits
            float pm = fmaxf(fmaxf(out[0], out[1]), fmaxf(out[2], out[3]));
            if (pm > -INFINITY) {
              const float mn = fmaxf(m_run, pm);
              float acc = m_run > -INFINITY ? s_run * exp_nonpos(fminf(m_run - mn, 0.f)) : 0.f;
#pragma unroll
              for (int k = 0; k < 4; ++k) acc += ((ok >> k) & 1u) ? exp_nonpos(fminf(lg[k] - mn, 0.f)) : 0.f;
              s_run = acc;
              m_run = mn;
            }
            if (!REPLAY) {
              uint32_t wd[4];
              philox4x32_10_ukey((uint32_t)sb, (uint32_t)t, (uint32_t)(64 * page + c), p.iter_lo, p.seed_lo, p.seed_hi, wd);
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                // Gumbel noise -log(-log u) from two hardware base-2 logarithms
                const float tl = -__builtin_amdgcn_logf(uniform_from_bits(wd[k]));                 // -log2 u > 0
                const float gn = -0.693147180559945f * __builtin_amdgcn_logf(tl) + 0.366512920581664f;  // - ln ln 2
                const float y = lg[k] + gn;
                const unsigned long long key =
                    ((unsigned long long)(~float_order(y)) << 32) | (uint32_t)(a0 + k);
                if (((ok >> k) & 1u) && key < best && given < 0) { best = key; l_best = lg[k]; }
              }
            }
            if (REPLAY || given >= 0) {
#pragma unroll
              for (int k = 0; k < 4; ++k)
                if (a0 + k == given) l_best = lg[k];
            }
          }
        }
      }

      // ================= SU: the lanes of a slot meet
      if (running) {
        const float M = grp32_max(m_run);
        const float S = grp32_sum(m_run > -INFINITY ? s_run * exp_nonpos(fminf(m_run - M, 0.f)) : 0.f);
        const float lse = M + __builtin_amdgcn_logf(S) * 0.693147180559945f;
        int act;
        bool given_ok = true;
        if (!REPLAY) {
          best = grp32_min_u64(best);
          act = given >= 0 ? given : (int)(uint32_t)best;
        } else {
          act = given;
          given_ok = act < A && (((myfill >> (act >> kb)) & 1u) == 0u);
          if (!given_ok) act = 0;
        }
        const float alogit = __shfl(l_best, ((act & 255) >> 2) & 31, 32);
        const int pos = act >> kb, word = act & (nw - 1);
        if (given_ok) {
          lpf += alogit - lse;
          lpb -= __builtin_amdgcn_logf((float)(t + 1)) * 0.693147180559945f;
        }
        if (si == 0) {
          p.lsebuf[myrow] = given_ok ? lse : __builtin_nanf("");
          if (!REPLAY) p.actions[myrow] = (uint16_t)act;
        }
        bool term = false;
        float logr = 0.f;
        if (!given_ok) {
          term = true;  // impossible action in the given sequence: the trajectory is cut here, state unchanged
        } else {
          if (t == Lp - 1) {
            int dmin = 0x7fffffff;
            for (int mm = si; mm < e.n_modes; mm += 32) {
              int dist = 0;
              for (int q = 0; q < Lp; ++q) {
                const uint32_t tok = (q == pos) ? (uint32_t)word : (uint32_t)words[sj * 32 + q];
                const uint32_t rev = __brev(tok) >> (32 - kb);
                dist += __popc(rev ^ mode_chunk(e.modes, e.words, mm, q, kb));
              }
              dmin = min(dmin, dist);
            }
            dmin = grp32_min(dmin);
            logr = -(e.beta / (float)e.n_bits) * (float)dmin;
            term = true;
          }
        }
        if (REPLAY) term = term || (t + 1 >= len_given);
        if (term) {
          if (si == 0) {
            if (!REPLAY) p.length[sb] = t + 1;
            p.lpf[sb] = lpf;
            p.lpb[sb] = lpb;
            p.logr[sb] = logr;
          }
          for (int s = si; s < Lp; s += 32) {
            int v = (s == pos && given_ok) ? word : (((myfill >> s) & 1u) ? (int)words[sj * 32 + s] : 0);
            p.term[(size_t)s * B + sb] = (int8_t)v;
          }
          running = false;
        }
        if (given_ok && si == 0) {
          words[sj * 32 + pos] = (uint8_t)word;
          filled[sj] = myfill | (1u << pos);
        }
      }
      lds_barrier();
    }
  }
}

// Turns the stored logits of every live transition into the direction of the logit gradient, in place:
// e[a] = [a = action taken] - exp(l_a - lse), 0 where the action was masked (l_a = -inf) and on rows whose
// log-sum-exp is NaN.  One workgroup of 256 threads per row of the list of live rows.
__global__ __launch_bounds__(256) void wide_logit_grad_kernel(float* __restrict__ lg, const float* __restrict__ lse,
                                                              const uint16_t* __restrict__ actions, int A,
                                                              const int* __restrict__ rows,
                                                              const int* __restrict__ hdr) {
  const int n = hdr[kHdrNLive];
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const int row = rows[i];
    const float ls = lse[row];
    const int act = actions[row];
    float* dst = lg + (size_t)row * A;
    for (int a0 = 4 * threadIdx.x; a0 < A; a0 += 1024) {
      const f32x4 l = *(const f32x4*)&dst[a0];
      f32x4 ev;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float pr = (l[k] > -INFINITY) ? __expf(l[k] - ls) : 0.f;
        ev[k] = (ls == ls) ? ((a0 + k == act ? 1.f : 0.f) - pr) : 0.f;
      }
      *(f32x4*)&dst[a0] = ev;
    }
  }
}

}  // namespace gfnx

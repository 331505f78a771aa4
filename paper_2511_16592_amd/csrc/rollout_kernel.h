// Persistent trajectory-block rollout kernel.
//
// One workgroup (8 wavefronts, two per SIMD) runs kSlots = 16 trajectories at a time from s_0 to their
// terminal states; it owns a contiguous range of p.tpw trajectories and a slot whose trajectory has ended
// starts the next one of the range (trajectory b is a pure function of (seed, iteration, b), so which slot
// runs it changes nothing).  Per step:
//   L2  hidden layer 2 on the matrix cores, computed transposed: D[feature][slot] = W2^T * relu(z1); the
//       eight waves split the output features; weights are MFMA A-operands (resident in registers when the
//       layer is 256 x 256: 128 registers per lane, or streamed from L2 cache in operand order with the next
//       step's loads in flight), activations come from LDS in B-operand order; on grids, a workgroup left with
//       at most four running trajectories (the tail of a batch of unequal walks) switches to the 4x4x1 matrix
//       instruction, which contracts the same resident operands against four slots at a quarter of the cost;
//   L3  logits the same way: output tiles split over the waves, and the contraction split as well when there
//       are fewer than eight tiles;
//   SU  per slot, 16 (grids) or 32 lanes of one wave: action mask, softmax weights, Philox draw and argmin by DPP row
//       rotations plus one swizzle, log P_F / log P_B, the row of the logit gradient, environment
//       transition, terminal log-reward, action byte; then the same lanes update the layer-1
//       pre-activation: layer 1 is a one-hot gather and a transition swaps exactly one active row, so z1 is
//       kept in LDS in binary64 and updated as z1 += (W1[new] - W1[old]), the difference rows prepared once per
//       rollout in binary64; what the matrix phase reads is h1 = relu((float)z1), written next to it.
// The post-ReLU activations h1, h2, their sign masks (1 bit per unit; those of h2 only where the gradient pass
// reads them), the state bytes and the logit-gradient direction (onehot(a) - p) of every transition are written to
// HBM rows t*B + b for the gradient pass.  Nothing the kernel writes to global memory is read back by it, so the
// two (single logit tile) or three barriers per step order LDS traffic only (no wait for stores to land).
#pragma once
#include "gfnx_device.h"

namespace gfnx {

constexpr int kRolloutWaves = 8;
constexpr int kRolloutThreads = 64 * kRolloutWaves;

template <int ENV>
__device__ __forceinline__ int initial_row(const EnvParams& e, int s) {
  if (ENV == 0) return e.H * s;
  if (ENV == 1 || ENV == 3) return ((1 << e.k_bits) + 1) * s + (1 << e.k_bits);
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

// max(v, 0) on the bit pattern: a negative float is a negative integer, a positive one keeps its order (one
// integer instruction, no canonicalisation of the operand)
__device__ __forceinline__ float relu1(float v) {
  return __builtin_bit_cast(float, max(__builtin_bit_cast(int, v), 0));
}
__device__ __forceinline__ f32x4 relu4(f32x4 v) {
  v.x = relu1(v.x); v.y = relu1(v.y); v.z = relu1(v.z); v.w = relu1(v.w);
  return v;
}

// Sign mask of 256 activations held four per lane (lane l: features 4l .. 4l+3): word k (k < 4) gets bit l
// set iff feature 4l+k is positive.  This is the ReLU derivative the gradient pass needs, at 1 bit per unit.
__device__ __forceinline__ void store_sign_mask(unsigned long long* dst, f32x4 v, int lane) {
  const unsigned long long m0 = __ballot(v.x > 0.f), m1 = __ballot(v.y > 0.f);
  const unsigned long long m2 = __ballot(v.z > 0.f), m3 = __ballot(v.w > 0.f);
  if (lane == 0) {  // dst is 32-byte aligned: rows hold a multiple of four words
    ((ulonglong2*)dst)[0] = make_ulonglong2(m0, m1);
    ((ulonglong2*)dst)[1] = make_ulonglong2(m2, m3);
  }
}

// exp(x) for x <= 0 on the transcendental unit: 2^(x log2 e) with the rounding error of the product fed back as a
// first-order correction; relative error below 2e-7 down to x = -40 (measured over 2^23 arguments), results under
// 2^-126 flush to zero.
__device__ __forceinline__ float exp_nonpos(float x) {
  const float t = x * 1.44269504088896341f;
  const float lo = __builtin_fmaf(x, 1.44269504088896341f, -t) + x * 1.92596299e-8f;
  const float e = __builtin_amdgcn_exp2f(t);
  return __builtin_fmaf(e, lo * 0.693147180559945f, e);
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

// (two accumulators per tile: an 8-cycle instruction leaves too little distance between dependent ones otherwise)
#define GFNX_MFMA4S(ACC, AV, BV)                                                           \
  ACC = __builtin_amdgcn_mfma_f32_4x4x1f32((AV).x, (BV).x, ACC, 0, 0, 0);                    \
  ACC##b = __builtin_amdgcn_mfma_f32_4x4x1f32((AV).y, (BV).y, ACC##b, 0, 0, 0);              \
  ACC = __builtin_amdgcn_mfma_f32_4x4x1f32((AV).z, (BV).z, ACC, 0, 0, 0);                    \
  ACC##b = __builtin_amdgcn_mfma_f32_4x4x1f32((AV).w, (BV).w, ACC##b, 0, 0, 0)

constexpr int kW2RegQ = 12;  // contraction steps (of 16) of a resident W2 tile held in registers; the rest sit in LDS

// Byte offsets of the kernel's LDS regions (shared by the launch code, which sizes the allocation).
struct RolloutLds {
  int h1s, h1s2, z1d, h2s, lgs, z1i, flags, st, ulog, w2l, total;
};
constexpr int kPitchD = 66;  // doubles per feature-quad row of the binary64 z1 tile (16 slots * 4 + 2 pad: conflict-free)
// rows2: h1 is double-buffered (read by the step in progress, written for the next one)
__host__ __device__ inline RolloutLds rollout_lds_layout(int H1, int H2, int A16, int SBL, bool stat, bool rows2) {
  const int ks = logits_ksplit(A16 >> 4, H2 >> 4);
  RolloutLds L;
  int o = 0;
  L.h1s = o; o += (H1 >> 2) * kPitch * 4;            // h1 = relu(z1) in binary32, B-operand order
  L.h1s2 = rows2 ? o : L.h1s; if (rows2) o += (H1 >> 2) * kPitch * 4;
  L.z1d = o; o += (H1 >> 2) * kPitchD * 8;           // pre-activation of layer 1 in binary64
  L.h2s = o; o += (H2 >> 2) * kPitch * 4;
  L.lgs = o; o += ks * (A16 >> 2) * kPitch * 4;      // [KS][A16 / 4] partial logits
  L.z1i = o; o += H1 * 8;                            // z1(s_0) in binary64, for slots that restart
  L.flags = o; o += (2 * kSlots + 4) * 4;            // srow[kSlots], qnext, live, (pad), utag[kSlots]
  L.st = o; o += kSlots * SBL;                       // state bytes, SBL per slot (a multiple of 16)
  L.ulog = o; if (rows2 && A16 == 16) o += kSlots * 4 * 16;  // draws made ahead: -log2(u) of 16 actions per slot
  L.w2l = o; if (stat) o += (16 - kW2RegQ) * 16 * 64 * 16;  // 16 tiles x (16 - kW2RegQ) steps x 64 lanes x 16 bytes
  L.total = o;
  return L;
}

// ENV  = 0 hypergrid, 1 bit sequences left to right, 2 Ising, 3 bit sequences in the non-autoregressive scheme.
// NTW  = 16-feature tiles of layer 2 per wave, ceil(H2 / 128).
// STAT = layer 2 is 256 x 256: each wave keeps its two tiles of W2 (32 KiB) on chip for the whole rollout,
//        kW2RegQ/16 of them in registers and the rest in LDS; with a single logit tile (grids) its eighth of
//        W3 as well.
// NCH  = chunks of four logits a lane may own in SU: 1 up to 128 actions, else 2.
// EXPLORE = epsilon-uniform exploration compiled in (free-running rollouts with epsilon > 0 only).
// CA16 = the padded number of logits when it is known at compile time (16: narrow grids, the shape whose per-step
//        latency matters most), 0 = taken from the parameters.
template <int ENV, bool REPLAY, int NTW, bool STAT, int NCH, bool EXPLORE, int CA16>
__global__ __launch_bounds__(kRolloutThreads) void rollout_kernel(const RolloutParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const EnvParams& e = p.env;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int g = lane >> 4, j16 = lane & 15;
  const int H1 = STAT ? 256 : p.H1, H2 = STAT ? 256 : p.H2;
  const int A = p.A, A16 = CA16 ? CA16 : p.A16, B = p.B, SBL = p.SBL;
  const int Q1 = H1 >> 4, Q2 = H2 >> 4;
  const int NT2 = H2 >> 4, NT3 = A16 >> 4, nchunk = A16 >> 2;
  const int KS = logits_ksplit(NT3, Q2);

  const RolloutLds L = rollout_lds_layout(H1, H2, A16, SBL, STAT, ENV == 0 && STAT);
  float* z1a = (float*)(smem_raw + L.h1s);
  float* z1b = (float*)(smem_raw + L.h1s2);
  double* z1d = (double*)(smem_raw + L.z1d);
  float* h2s = (float*)(smem_raw + L.h2s);
  float* lgs = (float*)(smem_raw + L.lgs);
  double* z1i = (double*)(smem_raw + L.z1i);
  int* srow = (int*)(smem_raw + L.flags);     // [kSlots] row t*B + b of the slot's current transition
  int* qnext = srow + kSlots;                 // next trajectory of this workgroup's range to start
  uint32_t* live = (uint32_t*)(qnext + 1);    // bit j: slot j is running a trajectory
  int* utag = srow + kSlots + 4;              // [kSlots] row index (t*B + b) the draws in `ulog` were made for
  f32x4* ulog = (f32x4*)(smem_raw + L.ulog);  // [kSlots][4 chunks] -log2(u) of the slot's next step
  int8_t* st = (int8_t*)(smem_raw + L.st);
  const f32x4* w2l = (const f32x4*)(smem_raw + L.w2l);

  const int b0 = blockIdx.x * p.tpw;                    // this workgroup's trajectories: [b0, bend)
  const int bend = min(B, b0 + p.tpw);
  // roles in the SU phase: LPS lanes (sub-lane si) of one wave per slot sj.  Grids have at most 32 logits, so 16
  // lanes per slot are enough and four waves (one per SIMD, with the vector unit to itself) serve all slots.
  // Grids with the resident layer 2: steps with at most kTailSlots running trajectories take the four-slot path
  // Grids: SU occupies four of the eight waves, so the other four write the h1 rows and sign masks of the step during
  // SU instead of all eight doing it at the head of the L2 phase.  They read the z1 the step was computed from while
  // SU writes the next one, hence the two buffers (z1a / z1b, swapped every step; one buffer otherwise).
  constexpr bool kRowsInSU = ENV == 0 && STAT;
  constexpr bool kTail = STAT && ENV == 0;
  // Narrow grids, free-running: the random draws of a step do not depend on the logits, so the four waves that are
  // not in SU make them one step ahead -- Philox and -log2(u) for the slot's next step, assuming its trajectory
  // goes on -- and SU takes them from LDS when they are for its (trajectory, step), else draws them itself.
  constexpr bool kDrawAhead = kRowsInSU && !REPLAY && CA16 == 16;
  constexpr int kTailSlots = 4;
  constexpr int LPS = ENV == 0 ? 16 : 32;
  constexpr int kSuWaves = kSlots / (64 / LPS);
  const int sj = (64 / LPS) * (w % kSuWaves) + lane / LPS, si = lane % LPS;
  const bool su_wave = w < kSuWaves;
  int8_t* stj = st + sj * SBL;                          // this slot's state bytes
  int sb = b0 + sj;                                     // trajectory in this slot
  int ts = 0;                                           // its step counter

  // ---- reset: s_0, z1(s_0) = b1 + sum of the initially active rows
  for (int f = tid; f < H1; f += kRolloutThreads) {
    double z = (double)p.b1[f];
    for (int s = 0; s < e.state_dim; ++s) z += (double)p.W1[(size_t)initial_row<ENV>(e, s) * H1 + f];
    const float h = relu1((float)z);
    float* dh = z1a + (f >> 2) * kPitch + (f & 3);
    float* dh2 = z1b + (f >> 2) * kPitch + (f & 3);
    double* dz = z1d + (f >> 2) * kPitchD + (f & 3);
#pragma unroll
    for (int j = 0; j < kSlots; ++j) { dh[j * 4] = h; dh2[j * 4] = h; dz[j * 4] = z; }
    z1i[f] = z;
  }
  for (int i = tid; 4 * i < SBL * kSlots; i += kRolloutThreads) ((uint32_t*)st)[i] = 0u;
  if (tid < kSlots) { srow[tid] = b0 + tid; utag[tid] = -1; }
  if (tid == 0) {
    *qnext = b0 + kSlots;
    const int n0 = bend - b0;  // at least one: the grid has no empty workgroup
    *live = n0 >= kSlots ? 0xFFFFu : ((1u << n0) - 1u);
  }
  float lpf = 0.f, lpb = 0.f;
  int len_given = 0;
  if (REPLAY && sb < bend) len_given = p.length[sb];
  f32x4 w2r[STAT ? 2 : 1][STAT ? kW2RegQ : 1];
  f32x4 w3r[STAT ? 2 : 1];
  if constexpr (STAT) {
    const f32x4* wp = (const f32x4*)p.W2p + (size_t)(w * 2) * 16 * 64 + lane;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
#pragma unroll
      for (int q = 0; q < kW2RegQ; ++q) w2r[n][q] = wp[(n * 16 + q) * 64];
#pragma unroll
      for (int q = kW2RegQ; q < 16; ++q)
        ((f32x4*)w2l)[((w * 2 + n) * (16 - kW2RegQ) + (q - kW2RegQ)) * 64 + lane] = wp[(n * 16 + q) * 64];
    }
    const f32x4* wp3 = (const f32x4*)p.W3p + lane;  // tile 0, this wave's eighth of the contraction
#pragma unroll
    for (int q = 0; q < 2; ++q) w3r[q] = wp3[(w * 2 + q) * 64];
  }
  // bias of the layer-2 features this lane finishes in L2
  f32x4 b2r[NTW];
#pragma unroll
  for (int n = 0; n < NTW; ++n) b2r[n] = *(const f32x4*)&p.b2[16 * min(w * NTW + n, NT2 - 1) + 4 * g];
  // bias of the logits this lane owns in the SU phase
  f32x4 b3r[NCH];
#pragma unroll
  for (int n = 0; n < NCH; ++n) {
    const int c = si + LPS * n;
#pragma unroll
    for (int k = 0; k < 4; ++k) b3r[n][k] = (c < nchunk && 4 * c + k < A) ? p.b3[4 * c + k] : 0.f;
  }
  // partial logits of a split contraction are summed across lanes when (parts x chunks) is exactly the 32
  // lanes of a slot (1, 2 or 4 logit tiles); otherwise by the owning lane
  const bool lane_sum = KS > 1 && KS * nchunk == 32;
  // Every register loaded above is read here once, so the wait for those loads sits before the step loop: inside
  // the loop a wait placed at their first use would also wait for the kernel's own recent stores each step.
#pragma unroll
  for (int n = 0; n < (STAT ? 2 : 1); ++n)
#pragma unroll
    for (int q = 0; q < (STAT ? kW2RegQ : 1); ++q) asm volatile("" ::"v"(w2r[n][q]));
#pragma unroll
  for (int n = 0; n < (STAT ? 2 : 1); ++n) asm volatile("" ::"v"(w3r[n]));
#pragma unroll
  for (int n = 0; n < NTW; ++n) asm volatile("" ::"v"(b2r[n]));
#pragma unroll
  for (int n = 0; n < NCH; ++n) asm volatile("" ::"v"(b3r[n]));
  lds_barrier();

  // list-scheduling bound on the number of steps: (sum of lengths) / kSlots + longest trajectory
  const int max_iters = e.max_steps * ((p.tpw + kSlots - 1) / kSlots + 1);
  for (int iter = 0; iter < max_iters; ++iter) {
    // ---- the running slots (one word, the same in every lane: kept on the scalar unit) and the row indices of this
    // step: of the two slots whose h1 / h2 rows this wave writes out and of the slot this lane serves in L2
    int sa[2], sr[2];
    int my_alive, my_row, su_alive;
    const uint32_t live_mask = __builtin_amdgcn_readfirstlane(*live);
    if (live_mask == 0u) break;
    sa[0] = (live_mask >> w) & 1u; sa[1] = (live_mask >> (w + 8)) & 1u;
    sr[0] = srow[w]; sr[1] = srow[w + 8];
    my_alive = (live_mask >> j16) & 1u; my_row = srow[j16];
    su_alive = (live_mask >> sj) & 1u;
    const float* z1s = (iter & 1) ? z1b : z1a;  // h1 of this step
    float* z1n = (iter & 1) ? z1a : z1b;        // ... of the next one (the same buffer unless double-buffered)
    int srk[4];                                 // rows of the four slots a non-SU wave writes out on grids
#pragma unroll
    for (int k = 0; k < 4; ++k) srk[k] = kRowsInSU ? srow[4 * (w & 3) + k] : 0;
    const int ahead_row = kDrawAhead ? srow[4 * (w & 3) + g] : 0;  // slot whose next draws this lane makes
    // ================= L2: h2 = relu(W2^T relu(z1) + b2)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {  // h1 rows and sign masks of slots w and w + 8
      if (kRowsInSU || !sa[hh]) continue;
      const int jj = w + 8 * hh;
      const size_t row = (size_t)sr[hh];
      float* dst = p.h1buf + row * H1;
      for (int it = 0; it * 64 < (H1 >> 2); ++it) {
        const int fg = lane + 64 * it;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (fg < (H1 >> 2)) {
          v = *(const f32x4*)&z1s[fg * kPitch + jj * 4];
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
        const f32x4* wl = w2l + (size_t)(w * 2) * (16 - kW2RegQ) * 64 + lane;
        // One contraction step; NEXT_READS = LDS reads of the following step (activations, plus the two weight
        // operands once past the register-resident part), which are issued before this step's eight matrix
        // instructions so that their latency is covered.  MFMA4 / SLOT: the matrix instruction and the slot whose
        // activations this lane feeds it.
#define GFNX_L2_STEP(NEXT_READS, MFMA4, SLOT, ACC0, ACC1)                                                      \
        {                                                                                            \
          const f32x4 bv = bvn;                                                                      \
          if (q + 1 < 16) bvn = *(const f32x4*)&z1s[(4 * (q + 1) + g) * kPitch + (SLOT) * 4];        \
          f32x4 a0, a1;                                                                              \
          if (q < kW2RegQ) {                                                                         \
            a0 = w2r[0][q];                                                                          \
            a1 = w2r[1][q];                                                                          \
          } else {                                                                                   \
            a0 = wl[(q - kW2RegQ) * 64];                                                             \
            a1 = wl[((16 - kW2RegQ) + (q - kW2RegQ)) * 64];                                          \
          }                                                                                          \
          MFMA4(ACC0, a0, bv);                                                                       \
          MFMA4(ACC1, a1, bv);                                                                       \
          __builtin_amdgcn_sched_group_barrier(0x100, NEXT_READS, 0);                                \
          __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                         \
        }
        bool tail = false;
        if constexpr (kTail) tail = __popc(live_mask) <= kTailSlots;  // the same in every wave
        if (tail) {
          // Four-slot path.  The 4x4x1 instruction multiplies, in each of 16 blocks of four lanes, a 4-vector of
          // A (one value per lane of the block) with a 4-vector of B: D[r] of lane l = A(lane 4 (l / 4) + r) * B(l).
          // Fed with the same resident W2 operands, lane l = 16 g + 4 m + j therefore accumulates, for the slot it
          // picks for j, units 16 tile + 4 m + r over the contraction indices of lane group g; the four groups
          // are summed across lanes, the four columns go to LDS and come back in the layout of the 16-slot path.
          // the (at most four) running slots, found on the scalar unit; lanes beyond their number repeat the first
          uint32_t wd = live_mask;
          const int s0 = __builtin_ctz(wd);
          wd &= wd - 1u;
          const int s1 = wd ? __builtin_ctz(wd) : s0;
          wd = wd ? (wd & (wd - 1u)) : 0u;
          const int s2 = wd ? __builtin_ctz(wd) : s0;
          wd = wd ? (wd & (wd - 1u)) : 0u;
          const int s3 = wd ? __builtin_ctz(wd) : s0;
          const int jj = lane & 3;
          const int sl = jj == 0 ? s0 : (jj == 1 ? s1 : (jj == 2 ? s2 : s3));  // jj-th running slot
          f32x4* part = (f32x4*)(h2s + 8 * w * kPitch);  // (the rows of the h2 tile that this wave owns)
          if (__popc(live_mask) == 1) {
            // One running slot (most steps of the longest walk of a batch): a matrix-vector product, which the vector
            // unit does in half the time the matrix instruction needs for its four columns.  Lane 16 g + u multiplies
            // the same resident operands (contraction indices of lane group g, unit 16 tile + u) with the slot's
            // activations, 128 multiply-adds in four chains, and leaves its partial sum where the four-slot path
            // leaves the column of its first slot.
            float p0a = 0.f, p0b = 0.f, p1a = 0.f, p1b = 0.f;
            // the activations are requested two steps ahead of their use, the LDS-resident weights one step ahead
            f32x4 hraw = *(const f32x4*)&z1s[(4 + g) * kPitch + s0 * 4];
            f32x4 hv = *(const f32x4*)&z1s[g * kPitch + s0 * 4];
#define GFNX_ONE_STEP(NEXT_READS)                                                                     \
            {                                                                                         \
              f32x4 hraw2 = hraw;                                                                     \
              if (q + 2 < 16) hraw2 = *(const f32x4*)&z1s[(4 * (q + 2) + g) * kPitch + s0 * 4];       \
              f32x4 a0, a1;                                                                           \
              if (q < kW2RegQ) {                                                                      \
                a0 = w2r[0][q];                                                                       \
                a1 = w2r[1][q];                                                                       \
              } else {                                                                                \
                a0 = wl[(q - kW2RegQ) * 64];                                                          \
                a1 = wl[((16 - kW2RegQ) + (q - kW2RegQ)) * 64];                                       \
              }                                                                                       \
              p0a = __builtin_fmaf(a0.x, hv.x, p0a); p1a = __builtin_fmaf(a1.x, hv.x, p1a);           \
              p0b = __builtin_fmaf(a0.y, hv.y, p0b); p1b = __builtin_fmaf(a1.y, hv.y, p1b);           \
              p0a = __builtin_fmaf(a0.z, hv.z, p0a); p1a = __builtin_fmaf(a1.z, hv.z, p1a);           \
              p0b = __builtin_fmaf(a0.w, hv.w, p0b); p1b = __builtin_fmaf(a1.w, hv.w, p1b);           \
              hv = hraw;                                                                              \
              hraw = hraw2;                                                                           \
              __builtin_amdgcn_sched_group_barrier(0x100, NEXT_READS, 0);                             \
              __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                                      \
            }
#pragma unroll
            for (int q = 0; q < kW2RegQ - 1; ++q) GFNX_ONE_STEP(1)
#pragma unroll
            for (int q = kW2RegQ - 1; q < 14; ++q) GFNX_ONE_STEP(3)
            {
              constexpr int q = 14;
              GFNX_ONE_STEP(2)
            }
            {
              constexpr int q = 15;
              GFNX_ONE_STEP(0)
            }
#undef GFNX_ONE_STEP
            float* pf = (float*)part;
            pf[4 * (16 * g + (j16 & ~3)) + (j16 & 3)] = p0a + p0b;         // [tile 0][g][unit quad][slot 0], element unit % 4
            pf[4 * (64 + 16 * g + (j16 & ~3)) + (j16 & 3)] = p1a + p1b;    // [tile 1] ...
          } else {
          // The 4x4x1 instruction occupies the pipe for 8 cycles, so the activations are requested two contraction
          // steps (128 cycles of matrix work) ahead of their use, and dependent instructions are four apart: the
          // two accumulators of a tile alternate, and the two tiles alternate inside each pair.
          f32x4 ta0 = {0.f, 0.f, 0.f, 0.f}, ta0b = ta0, ta1 = ta0, ta1b = ta0;
          f32x4 raw1 = *(const f32x4*)&z1s[(4 + g) * kPitch + sl * 4];
          f32x4 bv = *(const f32x4*)&z1s[g * kPitch + sl * 4];
#define GFNX_TAIL_STEP(NEXT_READS)                                                                    \
          {                                                                                           \
            f32x4 raw2 = raw1;                                                                        \
            if (q + 2 < 16) raw2 = *(const f32x4*)&z1s[(4 * (q + 2) + g) * kPitch + sl * 4];          \
            f32x4 a0, a1;                                                                             \
            if (q < kW2RegQ) {                                                                        \
              a0 = w2r[0][q];                                                                         \
              a1 = w2r[1][q];                                                                         \
            } else {                                                                                  \
              a0 = wl[(q - kW2RegQ) * 64];                                                            \
              a1 = wl[((16 - kW2RegQ) + (q - kW2RegQ)) * 64];                                         \
            }                                                                                         \
            ta0 = __builtin_amdgcn_mfma_f32_4x4x1f32(a0.x, bv.x, ta0, 0, 0, 0);                       \
            ta1 = __builtin_amdgcn_mfma_f32_4x4x1f32(a1.x, bv.x, ta1, 0, 0, 0);                       \
            ta0b = __builtin_amdgcn_mfma_f32_4x4x1f32(a0.y, bv.y, ta0b, 0, 0, 0);                     \
            ta1b = __builtin_amdgcn_mfma_f32_4x4x1f32(a1.y, bv.y, ta1b, 0, 0, 0);                     \
            ta0 = __builtin_amdgcn_mfma_f32_4x4x1f32(a0.z, bv.z, ta0, 0, 0, 0);                       \
            ta1 = __builtin_amdgcn_mfma_f32_4x4x1f32(a1.z, bv.z, ta1, 0, 0, 0);                       \
            ta0b = __builtin_amdgcn_mfma_f32_4x4x1f32(a0.w, bv.w, ta0b, 0, 0, 0);                     \
            ta1b = __builtin_amdgcn_mfma_f32_4x4x1f32(a1.w, bv.w, ta1b, 0, 0, 0);                     \
            bv = raw1;                                                                                \
            raw1 = raw2;                                                                              \
            /* issue order: the LDS reads placed ahead (activations of step q + 2, LDS-resident weights of */ \
            /* step q + 1), then this step's eight matrix instructions */                               \
            __builtin_amdgcn_sched_group_barrier(0x100, NEXT_READS, 0);                               \
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                        \
          }
#pragma unroll
          for (int q = 0; q < kW2RegQ - 1; ++q) GFNX_TAIL_STEP(1)
#pragma unroll
          for (int q = kW2RegQ - 1; q < 14; ++q) GFNX_TAIL_STEP(3)
          {
            constexpr int q = 14;
            GFNX_TAIL_STEP(2)
          }
          {
            constexpr int q = 15;
            GFNX_TAIL_STEP(0)
          }
#undef GFNX_TAIL_STEP
          acc[0] = ta0 + ta0b;
          acc[1] = ta1 + ta1b;
          // The four partial sums (one per lane group g) meet in this wave's own 2 KiB of the h2 tile: every lane
          // writes its partial columns, [tile][g][unit quad m][slot jj] (linear in the lane index), and reads, in
          // the layout of the 16-slot path, the four parts of (unit quad g, slot j16): rank of slot j16 among the
          // running ones (a slot that is not running reads some running slot's column; its results are unused).
#pragma unroll
          for (int n = 0; n < 2; ++n) part[n * 64 + lane] = acc[n];
          }
          const int rk = min(__popc(live_mask & ((1u << j16) - 1u)), 3);
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's own columns, written above
#pragma unroll
          for (int n = 0; n < 2; ++n) {
            const f32x4* src = part + n * 64 + 4 * g + rk;
            acc[n] = (src[0] + src[16]) + (src[32] + src[48]);
          }
        } else {
          f32x4 bvn = *(const f32x4*)&z1s[g * kPitch + j16 * 4];
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // the read of step 0 above
#pragma unroll
          for (int q = 0; q < kW2RegQ - 1; ++q) GFNX_L2_STEP(1, GFNX_MFMA4, j16, acc[0], acc[1])
#pragma unroll
          for (int q = kW2RegQ - 1; q < 15; ++q) GFNX_L2_STEP(3, GFNX_MFMA4, j16, acc[0], acc[1])
          {
            constexpr int q = 15;
            GFNX_L2_STEP(0, GFNX_MFMA4, j16, acc[0], acc[1])
          }
        }
#undef GFNX_L2_STEP
      } else if (w * NTW < NT2) {
        // tiles w*NTW .. w*NTW+NTW-1 (clamped: a clamped tile is computed twice and stored once); the weights
        // stream from L2 cache in operand order, two contraction steps ahead of their use
        const f32x4* wp = (const f32x4*)p.W2p + lane;
        const f32x4* wt[NTW];
#pragma unroll
        for (int n = 0; n < NTW; ++n) wt[n] = wp + (size_t)min(w * NTW + n, NT2 - 1) * Q1 * 64;
        f32x4 r[2][NTW];
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
          for (int n = 0; n < NTW; ++n) r[d][n] = wt[n][min(d, Q1 - 1) * 64];
        f32x4 bvn = *(const f32x4*)&z1s[g * kPitch + j16 * 4];
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
            bvn = *(const f32x4*)&z1s[(4 * min(q + 1, Q1 - 1) + g) * kPitch + j16 * 4];
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
      }
      if constexpr (STAT) {
        // This lane holds h2 of slot j16 for units 16 nt + 4 g .. + 3 of its two tiles: the row piece and its share
        // of the sign masks go to HBM from registers (unit 16 nt + 4 g + r is bit 4 (nt % 2) + g of byte nt / 2
        // = w of mask word r: one byte per slot, word and wave).
        f32x4 hv[2];
#pragma unroll
        for (int n = 0; n < 2; ++n) hv[n] = relu4(acc[n] + b2r[n]);
        const int alv = my_alive;
        const size_t row = (size_t)my_row;
#pragma unroll
        for (int n = 0; n < 2; ++n)
          if (alv) *(f32x4*)&p.h2buf[row * 256 + 16 * (2 * w + n) + 4 * g] = hv[n];
        if (p.m2buf) {  // (no consumer when the gradient pass takes the ReLU derivative from h2 itself)
          unsigned long long bal[2][4];
#pragma unroll
          for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int r = 0; r < 4; ++r) bal[n][r] = __ballot(alv && hv[n][r] > 0.f);
          // lane (j16, g) assembles the byte of mask word r = g: bit 4 n + g' comes from lane 16 g' + j16 of tile n
          uint32_t byte = 0;
#pragma unroll
          for (int n = 0; n < 2; ++n) {
            const unsigned long long b =
                g == 0 ? bal[n][0] : (g == 1 ? bal[n][1] : (g == 2 ? bal[n][2] : bal[n][3]));
            const unsigned long long x = b >> j16;
            const uint32_t nib = (uint32_t)(x & 1ull) | (uint32_t)((x >> 15) & 2ull) | (uint32_t)((x >> 30) & 4ull) |
                                 (uint32_t)((x >> 45) & 8ull);
            byte |= nib << (4 * n);
          }
          if (alv) ((uint8_t*)p.m2buf)[(row * p.MW2 + g) * 8 + w] = (uint8_t)byte;
        }
        if (NT3 == 1) {
          // a single logit tile (grids): the contraction is split by wave, and wave w's part runs over exactly
          // the 32 units it has just produced - the logits phase needs no LDS round trip and no barrier
          f32x4 acc3 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int n = 0; n < 2; ++n) { GFNX_MFMA4(acc3, w3r[n], hv[n]); }
          *(f32x4*)&lgs[(w * nchunk + g) * kPitch + j16 * 4] = acc3;
        } else {
#pragma unroll
          for (int n = 0; n < 2; ++n) *(f32x4*)&h2s[(4 * (2 * w + n) + g) * kPitch + j16 * 4] = hv[n];
        }
      } else {
#pragma unroll
        for (int n = 0; n < NTW; ++n) {
          const int nt = w * NTW + n;
          if (nt < NT2) *(f32x4*)&h2s[(4 * nt + g) * kPitch + j16 * 4] = relu4(acc[n] + b2r[n]);
        }
      }
    }
    // draws made ahead for this step: read before the barrier, since the other waves overwrite them during SU
    f32x4 ul_ahead = {0.f, 0.f, 0.f, 0.f};
    int ul_tag = -1;
    if (kDrawAhead && su_wave) {
      ul_ahead = ulog[sj * 4 + (si & 3)];
      ul_tag = utag[sj];
    }
    lds_barrier();

    // ================= L3: logits = W3^T h2 (+ b3 added in SU)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {  // (the resident-W2 variant has written h2 out of registers above)
      if (STAT || !sa[hh]) continue;
      const int jj = w + 8 * hh;
      const size_t row = (size_t)sr[hh];
      float* dst = p.h2buf + row * H2;
      for (int it = 0; it * 64 < (H2 >> 2); ++it) {
        const int fg = lane + 64 * it;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (fg < (H2 >> 2)) {
          v = *(const f32x4*)&h2s[fg * kPitch + jj * 4];
          *(f32x4*)&dst[fg * 4] = v;
        }
        if (p.m2buf) store_sign_mask(p.m2buf + (row * p.MW2 + 4 * it), v, lane);
      }
    }
    const bool logits_done = STAT && NT3 == 1;  // computed at the end of L2 above
    if (logits_done) {
    } else if (ENV != 0 && KS == 1) {
      // whole tiles: w and w + 8 (a wave without a second tile repeats its first: two independent accumulator
      // chains either way); the weights stream from L2 cache kL3Ahead contraction steps ahead of their use.
      // Grids have at most two logit tiles and never take this path.
      constexpr int kL3Ahead = 2;
      f32x4 acc[2];
#pragma unroll
      for (int n = 0; n < 2; ++n) acc[n] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (w < NT3) {
        const bool two = w + 8 < NT3;
        const f32x4* wp0 = (const f32x4*)p.W3p + (size_t)w * Q2 * 64 + lane;
        const f32x4* wp1 = (const f32x4*)p.W3p + (size_t)(two ? w + 8 : w) * Q2 * 64 + lane;
        f32x4 r0[kL3Ahead], r1[kL3Ahead];
#pragma unroll
        for (int d = 0; d < kL3Ahead; ++d) {
          r0[d] = wp0[min(d, Q2 - 1) * 64];
          r1[d] = wp1[min(d, Q2 - 1) * 64];
        }
        f32x4 bvn = *(const f32x4*)&h2s[g * kPitch + j16 * 4];
#pragma nounroll
        for (int q0 = 0; q0 < Q2; q0 += kL3Ahead) {  // Q2 is a multiple of 4 (hidden widths are multiples of 64)
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
            // issue order: the two weight loads kL3Ahead steps ahead, the next step's activations, then this
            // step's eight matrix instructions
            __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
          }
        }
        *(f32x4*)&lgs[(4 * w + g) * kPitch + j16 * 4] = acc[0];
        if (two) *(f32x4*)&lgs[(4 * (w + 8) + g) * kPitch + j16 * 4] = acc[1];
      }
    } else {
      // wave w: tile w / KS, contraction part w % KS
      const int nt = w / KS, ks = w - nt * KS;
      if (nt < NT3) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        const int qn = Q2 / KS;
        const f32x4* wp = (const f32x4*)p.W3p + lane;
        for (int q = ks * qn; q < (ks + 1) * qn; ++q) {
          const f32x4 bv = *(const f32x4*)&h2s[(4 * q + g) * kPitch + j16 * 4];
          const f32x4 av = wp[((size_t)nt * Q2 + q) * 64];
          GFNX_MFMA4(acc, av, bv);
        }
        *(f32x4*)&lgs[(ks * nchunk + 4 * nt + g) * kPitch + j16 * 4] = acc;
      }
    }
    if (!logits_done) lds_barrier();

    // ================= SU: mask, softmax, sample, bookkeeping, transition, z1 update (LPS lanes per slot)
    if (kRowsInSU && !su_wave) {
      // h1 rows and sign masks of this step, slots 4 (w - 4) .. + 3, while the other four waves are in SU
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int jj = 4 * (w & 3) + k;
        if (!((live_mask >> jj) & 1u)) continue;
        const size_t row = (size_t)srk[k];
        float* dst = p.h1buf + row * H1;
        for (int it = 0; it * 64 < (H1 >> 2); ++it) {
          const int fg = lane + 64 * it;
          f32x4 v = {0.f, 0.f, 0.f, 0.f};
          if (fg < (H1 >> 2)) {
            v = *(const f32x4*)&z1s[fg * kPitch + jj * 4];
            *(f32x4*)&dst[fg * 4] = v;
          }
          store_sign_mask(p.m1buf + (row * p.MW1 + 4 * it), v, lane);
        }
      }
      if constexpr (kDrawAhead) {
        const int dj = 4 * (w & 3) + g;  // 16 lanes per slot, as in SU; lane j16 < 4 owns chunk j16
        if (((live_mask >> dj) & 1u) && j16 < 4) {
          const int t1 = ahead_row / B + 1, b = ahead_row - (t1 - 1) * B;
          uint32_t wd[4];
          philox4x32_10_ukey((uint32_t)b, (uint32_t)t1, (uint32_t)j16, p.iter_lo, p.seed_lo, p.seed_hi, wd);
          f32x4 ul;
#pragma unroll
          for (int k = 0; k < 4; ++k) ul[k] = -__builtin_amdgcn_logf(uniform_from_bits(wd[k]));
          ulog[dj * 4 + j16] = ul;
          if (j16 == 0) utag[dj] = t1 * B + b;
        }
      }
    }
    if (su_wave && su_alive) {
      const int t = ts;
      // word si of the slot's state bytes: the validity bits of a grid lane's actions, and this lane's piece of
      // the state row kept for the gradient pass.  Read here, together with the partial logits below, so that the
      // phase starts with one round of LDS reads instead of a chain of them.
      const uint32_t stw = ((const uint32_t*)stj)[min(si, (SBL >> 2) - 1)];
      // ---- logits of this lane's chunks, validity bits, running maximum
      f32x4 lg[NCH];
      uint32_t vm[NCH];
      float m = -INFINITY;
#pragma unroll
      for (int n = 0; n < NCH; ++n) {
        const int c = si + LPS * n;
        f32x4 v = b3r[n];
        if (lane_sum) {
          // lane si holds part si / nchunk of chunk si % nchunk; the parts of a chunk are nchunk lanes apart
          f32x4 pv = *(const f32x4*)&lgs[si * kPitch + sj * 4];
          if (LPS == 16) pv += *(const f32x4*)&lgs[(si + 16) * kPitch + sj * 4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            float x = pv[k];
            if (LPS == 32) x += swz_xor16(x);
            if (nchunk <= 8) x += row16_rot<8>(x);
            if (nchunk <= 4) x += row16_rot<4>(x);
            pv[k] = x;
          }
          v += pv;
        } else if (c < nchunk) {
          for (int ks = 0; ks < KS; ++ks) v += *(const f32x4*)&lgs[(ks * nchunk + c) * kPitch + sj * 4];
        }
        lg[n] = v;
        // state bytes that decide the validity of actions 4c .. 4c+3, fetched as one word at a clamped index
        uint32_t sw = 0;
        if (ENV == 0) sw = stw;  // one chunk per lane on grids: c = si
        if (ENV == 2) sw = ((const uint16_t*)stj)[min(c, (SBL >> 1) - 1)];
        uint32_t bits = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int a = 4 * c + k;
          uint32_t ok;
          if (ENV == 0) {
            const int sv = (int)((sw >> (8 * k)) & 0xFFu);
            ok = (uint32_t)(a == e.d) | ((uint32_t)(a < e.d) & (uint32_t)(sv < e.H - 1));
          } else if (ENV == 1) {
            ok = (uint32_t)(a < A);
          } else if (ENV == 3) {
            // non-autoregressive bit sequences: action a writes to position a >> k; state byte 0 = empty
            const uint32_t sv = (uint8_t)stj[min(a >> e.k_bits, e.L - 1)];
            ok = (uint32_t)(a < A) & (uint32_t)(sv == 0u);
          } else {
            const uint32_t sv = (sw >> (8 * (k >> 1))) & 0xFFu;
            ok = (uint32_t)(a < A) & (uint32_t)(sv == 0u);
          }
          bits |= ok << k;
          m = fmaxf(m, ok ? v[k] : -INFINITY);
        }
        vm[n] = bits;
      }
      m = grp_max<LPS>(m);
      if (p.sbuf && 4 * si < p.SB)  // the state the policy is evaluated at (SB <= 4 LPS bytes, a multiple of 16)
        ((uint32_t*)(p.sbuf + ((size_t)t * B + sb) * p.SB))[si] = stw;
      // ---- softmax weights exp(l - m) of the valid actions (0 elsewhere) and their sum
      f32x4 wv[NCH];
      float sum = 0.f;
#pragma unroll
      for (int n = 0; n < NCH; ++n)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float ex = exp_nonpos(fminf(lg[n][k] - m, 0.f));
          wv[n][k] = ((vm[n] >> k) & 1u) ? ex : 0.f;
          sum += wv[n][k];
        }
      sum = grp_sum<LPS>(sum);
      // logarithm and reciprocal on the transcendental unit (1 ulp): log P_F accumulates errors of ~1e-7 per step
      const float lse = __builtin_amdgcn_logf(sum) * 0.693147180559945f;
      const float inv_sum = __builtin_amdgcn_rcpf(sum);

      int act;
      bool given_ok = true;  // teacher-forced mode: is the given action possible in this state?
      if (!REPLAY) {
        // Gumbel-max as an exponential race: argmax_a (l_a - log(-log u_a)) = argmin_a (-log u_a) / exp(l_a - m),
        // one logarithm per action (base 2: the common factor ln 2 does not move the argmin); logarithm and
        // reciprocal on the transcendental unit, relative error of the key below 4e-7.  An action of weight 0
        // (invalid, or underflowed) gets the key +inf and cannot win: the largest valid logit has weight 1.  Key
        // (a non-negative float, ordered like its bit pattern) and action index are packed into 64 bits, so one
        // unsigned minimum finds the winner and lets the lowest index win exact ties.
        unsigned long long best = ~0ull;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
          const int c = si + LPS * n;
          f32x4 ul;  // -log2(u) of the four actions
          if (kDrawAhead && ul_tag == t * B + sb) {
            ul = ul_ahead;  // (lanes beyond the four chunks hold a copy of one of them; their weights are 0)
          } else {
            uint32_t wd[4];
            philox4x32_10_ukey((uint32_t)sb, (uint32_t)t, (uint32_t)c, p.iter_lo, p.seed_lo, p.seed_hi, wd);
#pragma unroll
            for (int k = 0; k < 4; ++k) ul[k] = -__builtin_amdgcn_logf(uniform_from_bits(wd[k]));
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float r = ul[k] * __builtin_amdgcn_rcpf(wv[n][k]);
            const unsigned long long key =
                ((unsigned long long)__builtin_bit_cast(uint32_t, r) << 32) | (uint32_t)(4 * c + k);
            best = key < best ? key : best;
          }
        }
        best = grp_min_u64<LPS>(best);
        act = (int)(uint32_t)best;
        if constexpr (EXPLORE) {
          // epsilon-uniform exploration (Appendix "Bit sequences", experimental setting): one more Philox call
          // per step, counter (b, t, 0xFFFFFFFE, iteration); word 0 decides, the same in every lane of the slot;
          // word 1 picks the j-th valid action in increasing order, j = floor(w n / 2^32).  Chunks are owned in
          // the order (pass, lane), so the rank of a lane's first valid action is a prefix sum over the lanes.
          uint32_t we[4];
          philox4x32_10_ukey((uint32_t)sb, (uint32_t)t, 0xFFFFFFFEu, p.iter_lo, p.seed_lo, p.seed_hi, we);
          if (uniform_from_bits(we[0]) < p.eps) {
            int pre[NCH], cnt[NCH], total = 0;
#pragma unroll
            for (int n = 0; n < NCH; ++n) {
              cnt[n] = __popc(vm[n]);
              int incl = cnt[n];
#pragma unroll
              for (int d = 1; d < LPS; d <<= 1) {
                const int o = __shfl_up(incl, d, LPS);
                if (si >= d) incl += o;
              }
              pre[n] = total + incl - cnt[n];
              total += __shfl(incl, LPS - 1, LPS);
            }
            const int j = (int)__umulhi(we[1], (uint32_t)total);
            int cand = 0x7fffffff;
#pragma unroll
            for (int n = 0; n < NCH; ++n) {
              int jl = j - pre[n];
              if (jl >= 0 && jl < cnt[n]) {
                uint32_t bb = vm[n];
                int k = 0;
                const int c2 = __popc(bb & 3u);
                if (jl >= c2) { jl -= c2; k = 2; bb >>= 2; }
                if (jl >= (int)(bb & 1u)) k += 1;
                cand = 4 * (si + LPS * n) + k;
              }
            }
            act = grp_min<LPS>(cand);
          }
        }
      } else {
        act = p.actions[(size_t)t * B + sb];
      }
      // logit of the action taken, from the lane that owns it
      float alogit;
      {
        float mine = 0.f;
        int mine_ok = 0;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
          const bool own = (act >> 2) / LPS == n;  // chunk act / 4 = si + LPS n
          const int k = act & 3;
          const float x = k == 0 ? lg[n].x : (k == 1 ? lg[n].y : (k == 2 ? lg[n].z : lg[n].w));
          mine = own ? x : mine;
          mine_ok = own ? (int)((vm[n] >> k) & 1u) : mine_ok;
        }
        alogit = __shfl(mine, (act >> 2) % LPS, LPS);
        if (REPLAY) {
          given_ok = (act < A) && __shfl(mine_ok, (act >> 2) % LPS, LPS) != 0;
          if (!given_ok) { act = 0; alogit = m + lse; }  // log p = 0; the trajectory is cut below
        }
      }
      lpf += (alogit - m) - lse;
      // network with a flow output: output d + 1 is log F of the state the policy was evaluated at (never a valid
      // action: the validity bits of a grid stop at d); its owner lane hands it to the slot
      float phi_here = 0.f;
      if (ENV == 0 && p.phibuf) {
        const int fa = e.d + 1, fk = fa & 3;
        const float mine = fk == 0 ? lg[0].x : (fk == 1 ? lg[0].y : (fk == 2 ? lg[0].z : lg[0].w));
        phi_here = __shfl(mine, fa >> 2, LPS);
      }
      const float lpb_before = lpb;

      // the one-hot row that leaves / enters the input with this action (known to all lanes of the slot); the
      // two rows of W1 are requested now so that their latency overlaps the bookkeeping below
      int rold = 0, rnew = 0;
      if (!REPLAY || given_ok) {
        if (ENV == 0) {
          if (act != e.d) {
            rold = e.H * act + stj[act];
            rnew = rold + 1;
          }
        } else if (ENV == 1) {
          rold = ((1 << e.k_bits) + 1) * ts + (1 << e.k_bits);
          rnew = ((1 << e.k_bits) + 1) * ts + act;
        } else if (ENV == 3) {
          rold = ((1 << e.k_bits) + 1) * (act >> e.k_bits) + (1 << e.k_bits);
          rnew = ((1 << e.k_bits) + 1) * (act >> e.k_bits) + (act & ((1 << e.k_bits) - 1));
        } else {
          rold = 3 * (act >> 1) + 1;
          rnew = 3 * (act >> 1) + 2 * (act & 1);
        }
      }
      // pieces of the difference row W1[rnew] - W1[rold] (binary64, indexed by rnew) requested early: all of a
      // 256-wide layer
      constexpr int kPre = 64 / LPS;
      f64x2 da[kPre], db[kPre];
      (void)rold;
#pragma unroll
      for (int it = 0; it < kPre; ++it) {
        const int fg = min(si + LPS * it, (H1 >> 2) - 1);
        const f64x2* dp = (const f64x2*)&p.D1[(size_t)rnew * H1 + 4 * fg];
        da[it] = dp[0];
        db[it] = dp[1];
      }

      {  // direction of the logit gradient: onehot(a) - p on valid actions, 0 elsewhere (weight 0 there)
        float* erow = p.ebuf + ((size_t)t * B + sb) * A16;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
          const int c = si + LPS * n;
          if (c < nchunk) {
            f32x4 ev;
#pragma unroll
            for (int k = 0; k < 4; ++k) ev[k] = (4 * c + k == act ? 1.f : 0.f) - wv[n][k] * inv_sum;
            if (REPLAY && !given_ok) ev = (f32x4){0.f, 0.f, 0.f, 0.f};
            *(f32x4*)&erow[4 * c] = ev;
          }
        }
      }

      bool term = false;
      float logr = 0.f;
      int xi = 0;              // grid: this lane's coordinate after the step
      int site = 0, spin = 0;  // ising
      if (REPLAY && !given_ok) {
        term = true;  // impossible action in the given sequence: cut the trajectory here, state unchanged
        if (ENV == 0) xi = (si < e.d) ? stj[si] : 0;
        site = -1;
      } else if (ENV == 0) {
        xi = (si < e.d) ? stj[si] : 0;
        if (act != e.d) {
          if (si == act) { stj[si] = (int8_t)(xi + 1); xi += 1; }
          const int cnt = grp_sum<LPS>((si < e.d && xi > 0) ? 1 : 0);
          lpb -= __builtin_amdgcn_logf((float)cnt) * 0.693147180559945f;
        } else {
          // v = |x / (H-1) - 1/2| against the strict thresholds 1/4, 3/10 and 2/5 of the reward equation, decided on
          // integers (a coordinate sits exactly on a threshold whenever H-1 is a multiple of 4, 5 or 10):
          // 1/4 < v <=> H-1 < |4x - 2(H-1)|;  3/10 < v < 2/5 <=> 3(H-1) < |10x - 5(H-1)| < 4(H-1)
          const int hm = e.H - 1;
          const int q4 = abs(4 * xi - 2 * hm), q10 = abs(10 * xi - 5 * hm);
          const int bad1 = grp_sum<LPS>((si < e.d && !(hm < q4)) ? 1 : 0);
          const int bad2 = grp_sum<LPS>((si < e.d && !((3 * hm < q10) && (q10 < 4 * hm))) ? 1 : 0);
          const float r = e.r0 + e.r1 * (bad1 == 0 ? 1.f : 0.f) + e.r2 * (bad2 == 0 ? 1.f : 0.f);
          logr = __builtin_amdgcn_logf(r) * 0.693147180559945f;  // hardware log2: |error| ~1e-6 on |log R| <= 7
          term = true;
        }
      } else if (ENV == 1) {
        const int k = e.k_bits;
        if (si == 0) stj[t] = (int8_t)act;
        if (t == e.L - 1) {
          int dmin = 0x7fffffff;
          for (int mm = si; mm < e.n_modes; mm += LPS) {
            int dist = 0;
            for (int pos = 0; pos < e.L; ++pos) {
              const uint32_t tok = (pos == t) ? (uint32_t)act : (uint32_t)(uint8_t)stj[pos];
              const uint32_t rev = __brev(tok) >> (32 - k);
              dist += __popc(rev ^ mode_chunk(e.modes, e.words, mm, pos, k));
            }
            dmin = min(dmin, dist);
          }
          dmin = grp_min<LPS>(dmin);
          logr = -(e.beta / (float)e.n_bits) * (float)dmin;
          term = true;
        }
      } else if (ENV == 3) {
        // non-autoregressive bit sequences: `site` = position, `spin` = the k-bit word written there (state byte
        // word + 1, 0 = empty); the backward policy is uniform over the t+1 filled positions of the child
        const int k = e.k_bits;
        site = act >> k;
        spin = act & ((1 << k) - 1);
        if (si == 0) stj[site] = (int8_t)(spin + 1);
        lpb -= __builtin_amdgcn_logf((float)(t + 1)) * 0.693147180559945f;
        if (t == e.L - 1) {
          int dmin = 0x7fffffff;
          for (int mm = si; mm < e.n_modes; mm += LPS) {
            int dist = 0;
            for (int pos = 0; pos < e.L; ++pos) {
              const uint32_t tok = (pos == site) ? (uint32_t)spin : (uint32_t)(uint8_t)stj[pos] - 1u;
              const uint32_t rev = __brev(tok) >> (32 - k);
              dist += __popc(rev ^ mode_chunk(e.modes, e.words, mm, pos, k));
            }
            dmin = min(dmin, dist);
          }
          dmin = grp_min<LPS>(dmin);
          logr = -(e.beta / (float)e.n_bits) * (float)dmin;
          term = true;
        }
      } else {
        site = act >> 1;
        spin = 2 * (act & 1) - 1;
        if (si == 0) stj[site] = (int8_t)spin;
        lpb -= __builtin_amdgcn_logf((float)(t + 1)) * 0.693147180559945f;
        if (t == e.D - 1) {
          int acc = 0;
          for (int s = si; s < e.D; s += LPS) {
            const int r = s / e.N, c = s - r * e.N;
            const int sr = r * e.N + (c + 1 == e.N ? 0 : c + 1);
            const int sd = (r + 1 == e.N ? 0 : r + 1) * e.N + c;
            const int x = (s == site) ? spin : stj[s];
            const int xr = (sr == site) ? spin : stj[sr];
            const int xd = (sd == site) ? spin : stj[sd];
            acc += x * (xr + xd);
          }
          acc = grp_sum<LPS>(acc);
          logr = e.coupling * (float)acc;
          term = true;
        }
      }
      if (REPLAY) term = term || (t + 1 >= len_given);
      if (!REPLAY && si == 0) p.actions[(size_t)t * B + sb] = (uint8_t)act;
      if (ENV == 0 && p.phibuf && si == 0) {
        p.phibuf[(size_t)t * B + sb] = phi_here;
        p.dlbuf[(size_t)t * B + sb] = ((alogit - m) - lse) - (lpb - lpb_before);
      }
      if (term) {
        if (si == 0) {
          if (!REPLAY) p.length[sb] = t + 1;
          p.lpf[sb] = lpf;
          p.lpb[sb] = lpb;
          p.logr[sb] = logr;
        }
        for (int s = si; s < e.state_dim; s += LPS) {
          int v;
          if (ENV == 0) v = xi;  // state_dim <= 16: lane s holds coordinate s
          else if (ENV == 1) v = (s == t && given_ok) ? act : (int)(uint8_t)stj[s];
          else if (ENV == 3) v = (s == site) ? spin : (int)(uint8_t)stj[s] - 1;
          else v = (s == site) ? spin : stj[s];
          p.term[(size_t)s * B + sb] = (int8_t)v;
        }
        // the slot starts the next trajectory of the workgroup's range, if any is left
        int nb = 0;
        if (si == 0) nb = atomicAdd(qnext, 1);
        nb = __shfl(nb, 0, LPS);
        if (nb < bend) {
          sb = nb;
          ts = 0;
          lpf = 0.f;
          lpb = 0.f;
          if (REPLAY) len_given = p.length[sb];
          for (int s4 = si; 4 * s4 < SBL; s4 += LPS) ((uint32_t*)stj)[s4] = 0u;
          for (int fg = si; fg < (H1 >> 2); fg += LPS) {
            const f64x2 a = ((const f64x2*)&z1i[4 * fg])[0], b = ((const f64x2*)&z1i[4 * fg])[1];
            f64x2* zp = (f64x2*)&z1d[fg * kPitchD + sj * 4];
            zp[0] = a;
            zp[1] = b;
            *(f32x4*)&z1n[fg * kPitch + sj * 4] =
                (f32x4){relu1((float)a.x), relu1((float)a.y), relu1((float)b.x), relu1((float)b.y)};
          }
          if (si == 0) srow[sj] = sb;
        } else if (si == 0) {
          atomicAnd(live, ~(1u << sj));
        }
      } else {
        ts = t + 1;
        if (si == 0) srow[sj] = ts * B + sb;
        // z1 += W1[new row] - W1[old row] for this slot, in binary64 (the difference row comes prepared): however
        // long the walk, relu and its derivative see the correctly rounded sum of the active rows
        auto update = [&](int fg, f64x2 a, f64x2 b) {
          f64x2* zp = (f64x2*)&z1d[fg * kPitchD + sj * 4];
          const f64x2 z0 = zp[0] + a, z1 = zp[1] + b;
          zp[0] = z0;
          zp[1] = z1;
          *(f32x4*)&z1n[fg * kPitch + sj * 4] =
              (f32x4){relu1((float)z0.x), relu1((float)z0.y), relu1((float)z1.x), relu1((float)z1.y)};
        };
#pragma unroll
        for (int it = 0; it < kPre; ++it)
          if (si + LPS * it < (H1 >> 2)) update(si + LPS * it, da[it], db[it]);
        for (int fg = si + LPS * kPre; fg < (H1 >> 2); fg += LPS) {
          const f64x2* dp = (const f64x2*)&p.D1[(size_t)rnew * H1 + 4 * fg];
          update(fg, dp[0], dp[1]);
        }
      }
      // the difference rows were requested on every path but are consumed only when the trajectory goes on: read them
      // here, so that the wait for these loads (not for the stores issued after them) closes the phase and the
      // next phase does not start by waiting for everything outstanding
#pragma unroll
      for (int it = 0; it < kPre; ++it) asm volatile("" ::"v"(da[it]), "v"(db[it]));
    }
    lds_barrier();
  }
}

// Everything a rollout needs prepared from the weights, in one launch (block ranges of 128 / 256 / 64 / 512
// blocks of 256 threads; the last range writes the difference rows of layer 1, see difference_rows_part):
//   W2p, W3p  W[K][N] row-major -> MFMA A-operand order, out[nt][q][lane][s] = W[16q + 4*(lane/16) + s][16nt + lane%16],
//             zero beyond column N (the rollout's layer-2 and logit weights);
//   actions   every action byte <- 0xFF padding, as 32-bit words (the buffer is 4-byte aligned); skipped when null.
struct PrepareParams {
  const float *W1, *W2, *W3;
  int In, H1, H2, A, A16;
  float *W2p, *W3p;
  double* D1;       // [In][H1] difference rows of layer 1
  int kind, group;  // environment kind; one-hot columns per state component (grid side, 2^k + 1, 3)
  uint8_t* actions;
  size_t action_bytes;
};
// D1[r] = W1[r] - W1[old(r)] in binary64: the change of the layer-1 pre-activation when the transition makes one-hot
// row r active in place of row old(r) -- grid: r - 1 (the coordinate one lower; rows of coordinate 0 are never entered),
// bit sequences: the "empty" row of the position, Ising: the "unassigned" row of the site.
__device__ __forceinline__ void difference_rows_part(const PrepareParams& p, int block, int blocks) {
  const int qv = p.H1 >> 2;  // four columns per thread
  const size_t total = (size_t)p.In * qv;
  for (size_t i = (size_t)block * 256 + threadIdx.x; i < total; i += (size_t)blocks * 256) {
    const int r = (int)(i / qv), f = 4 * (int)(i - (size_t)r * qv);
    const int c = r / p.group, v = r - c * p.group;
    int ro;
    if (p.kind == 0) ro = v > 0 ? r - 1 : r;
    else if (p.kind == 1) ro = c * p.group + (p.group - 1);
    else ro = c * p.group + 1;
    const f32x4 a = *(const f32x4*)&p.W1[(size_t)r * p.H1 + f], b = *(const f32x4*)&p.W1[(size_t)ro * p.H1 + f];
    f64x2* d = (f64x2*)&p.D1[(size_t)r * p.H1 + f];
    d[0] = (f64x2){(double)a.x - (double)b.x, (double)a.y - (double)b.y};
    d[1] = (f64x2){(double)a.z - (double)b.z, (double)a.w - (double)b.w};
  }
}
__device__ __forceinline__ void pack_weights_part(const float* __restrict__ W, int K, int N, int NT,
                                                  float* __restrict__ out, int block, int blocks) {
  const int Q = K >> 4;
  const size_t total = (size_t)NT * Q * 256;
  for (size_t i = (size_t)block * 256 + threadIdx.x; i < total; i += (size_t)blocks * 256) {
    const int s = (int)(i & 3), ln = (int)((i >> 2) & 63);
    const size_t r = i >> 8;
    const int q = (int)(r % Q), nt = (int)(r / Q);
    const int k = 16 * q + 4 * (ln >> 4) + s, n = 16 * nt + (ln & 15);
    out[i] = n < N ? W[(size_t)k * N + n] : 0.f;
  }
}
constexpr int kDiffBlocks = 512;
constexpr int kPrepareBlocks = 128 + 256 + 64 + kDiffBlocks;
__global__ __launch_bounds__(256) void prepare_kernel(const PrepareParams p) {
  int b = blockIdx.x;
  if (b < 128) { pack_weights_part(p.W2, p.H1, p.H2, p.H2 >> 4, p.W2p, b, 128); return; }
  b -= 128;
  if (b < 256) { pack_weights_part(p.W3, p.H2, p.A, p.A16 >> 4, p.W3p, b, 256); return; }
  b -= 256;
  if (b >= 64) {
    if (p.D1) difference_rows_part(p, b - 64, kDiffBlocks);
    return;
  }
  if (p.actions) {
    const size_t words = p.action_bytes >> 2;
    for (size_t i = (size_t)b * 256 + threadIdx.x; i < words; i += (size_t)64 * 256) ((uint32_t*)p.actions)[i] = 0xFFFFFFFFu;
    if (b == 0 && threadIdx.x < (p.action_bytes & 3)) p.actions[(words << 2) + threadIdx.x] = 0xFF;
  }
}

}  // namespace gfnx

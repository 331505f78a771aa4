// Shared device-side definitions of libgfnx_hip: parameter blocks, MFMA wrappers, the counter-based
// RNG and small wavefront helpers.  gfx950 only (64-wide wavefronts, fp32 MFMA).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gfnx {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

constexpr int kSlots = 16;         // trajectories per workgroup of the rollout kernel (one MFMA N-tile)
constexpr int kPitch = 68;         // floats per feature-quad row of an activation tile in LDS (16 slots * 4 + 4 pad)
constexpr int kMaxStateDim = 100;  // largest state vector (Ising 10x10)

struct EnvParams {
  int kind;
  int d, H;  // grid
  float r0, r1, r2;
  int n_bits, k_bits, L, n_modes, words;  // bitseq
  const uint32_t* modes;
  float beta;
  int N, D;  // ising
  float coupling;
  int state_dim, obs_dim, n_actions, max_steps;
};

struct RolloutParams {
  EnvParams env;
  int In, H1, H2, A, A16;
  const float *W1, *b1, *b2, *b3;
  const float *W2p, *W3p;  // weights re-laid-out as MFMA A-operands
  const double* D1;        // [In][H1] difference rows of layer 1: W1[r] - W1[row that r replaces], binary64
  uint32_t seed_lo, seed_hi, iter_lo;
  int B, T;  // batch, traj.max_steps
  int tpw;   // trajectories owned by one workgroup (multiple of kSlots)
  uint8_t* actions;
  int* length;
  int8_t* term;
  float *lpf, *lpb, *logr;
  float *h1buf, *h2buf, *ebuf;  // per-transition rows, row = t*B + b
  unsigned long long *m1buf, *m2buf;  // sign masks of h1 / h2: MW1 / MW2 words of 64 bits per row
  int MW1, MW2;
  uint8_t* sbuf;  // state bytes of every transition (SB per row), or null when the gradient pass needs none
  int SB;
  int SBL;        // bytes per slot of the state kept in LDS: a multiple of 16, >= max(state_dim, SB)
  float eps;      // epsilon-uniform exploration: probability of a uniform draw over the valid actions (0 = off)
  // networks with a flow output (grids): log F(s_t) and log P_F - log P_B of every transition, row t*B + b; or null
  float *phibuf, *dlbuf;
};

// D(16x16) += A(16x4) * B(4x16).  Lane l supplies A[i = l%16][k = l/16] and B[k = l/16][j = l%16];
// it receives D[i = 4*(l/16) + r][j = l%16] in register r.
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
// D(32x32) += A(32x2) * B(2x32).  Lane l supplies A[i = l%32][k = l/32] and B[k = l/32][j = l%32];
// it receives D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32] in register r.
__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies,
// key bumped by the Weyl constants each round.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiply per product (high and low halves from the same instruction)
    const unsigned long long p0 = (unsigned long long)0xD2511F53u * (unsigned long long)c0;
    const unsigned long long p1 = (unsigned long long)0xCD9E8D57u * (unsigned long long)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The same with a wavefront-uniform key.  The round keys are bumped on the scalar unit as the rounds go; the empty
// asm keeps the compiler from precomputing all ten pairs outside the caller's loop, where they would occupy
// twenty scalar registers for the whole kernel.
__device__ __forceinline__ void philox4x32_10_ukey(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                   uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiply per product (high and low halves from the same instruction)
    const unsigned long long p0 = (unsigned long long)0xD2511F53u * (unsigned long long)c0;
    const unsigned long long p1 = (unsigned long long)0xCD9E8D57u * (unsigned long long)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
    asm volatile("" : "+s"(k0), "+s"(k1));
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 32 random bits -> u in (0,1), exactly representable in binary32
__device__ __forceinline__ float uniform_from_bits(uint32_t w) {
  return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f;  // 2^-23
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's LDS operations, not for its
// outstanding global stores (the kernels using it never read back what they store to global memory).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Value of the lane `n` positions further round the aligned row of 16 lanes (DPP row rotation).
// (every lane of a rotation has a source, so the "old" operand is left undefined: the move can then be folded into
// the instruction that consumes it)
template <int N>
__device__ __forceinline__ int row16_rot(int v) {
  return __builtin_amdgcn_mov_dpp(v, 0x120 + N, 0xF, 0xF, true);
}
template <int N>
__device__ __forceinline__ float row16_rot(float v) {
  return __builtin_bit_cast(float, row16_rot<N>(__builtin_bit_cast(int, v)));
}

// Reductions over the 16 lanes that serve one trajectory slot (an aligned quarter of a wavefront); every
// lane of the row ends with the same result.  All 16 lanes must be active together.
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, row16_rot<8>(v)); v = fmaxf(v, row16_rot<4>(v));
  v = fmaxf(v, row16_rot<2>(v)); v = fmaxf(v, row16_rot<1>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += row16_rot<8>(v); v += row16_rot<4>(v); v += row16_rot<2>(v); v += row16_rot<1>(v);
  return v;
}
__device__ __forceinline__ int row16_sum(int v) {
  v += row16_rot<8>(v); v += row16_rot<4>(v); v += row16_rot<2>(v); v += row16_rot<1>(v);
  return v;
}
__device__ __forceinline__ int row16_min(int v) {
  v = min(v, row16_rot<8>(v)); v = min(v, row16_rot<4>(v));
  v = min(v, row16_rot<2>(v)); v = min(v, row16_rot<1>(v));
  return v;
}
// (key, idx, payload) of the smallest key over the row; the lowest idx wins equal keys
template <int N>
__device__ __forceinline__ void row16_argmin_step(float& key, int& idx, float& payload) {
  const float ok = row16_rot<N>(key), op = row16_rot<N>(payload);
  const int oi = row16_rot<N>(idx);
  if (ok < key || (ok == key && oi < idx)) { key = ok; idx = oi; payload = op; }
}
__device__ __forceinline__ void row16_argmin(float& key, int& idx, float& payload) {
  row16_argmin_step<8>(key, idx, payload);
  row16_argmin_step<4>(key, idx, payload);
  row16_argmin_step<2>(key, idx, payload);
  row16_argmin_step<1>(key, idx, payload);
}

// ---- the same over 32 lanes (an aligned half of a wavefront): row reduction, then one exchange with the
// other row of the half through the swizzle network (lane i <-> lane i ^ 16)
__device__ __forceinline__ int swz_xor16(int v) { return __builtin_amdgcn_ds_swizzle(v, 0x401F); }
__device__ __forceinline__ float swz_xor16(float v) {
  return __builtin_bit_cast(float, swz_xor16(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ float grp32_max(float v) { v = row16_max(v); return fmaxf(v, swz_xor16(v)); }
__device__ __forceinline__ float grp32_sum(float v) { v = row16_sum(v); return v + swz_xor16(v); }
__device__ __forceinline__ int grp32_sum(int v) { v = row16_sum(v); return v + swz_xor16(v); }
__device__ __forceinline__ int grp32_min(int v) { v = row16_min(v); return min(v, swz_xor16(v)); }
// unsigned 64-bit minimum over the 32 lanes
template <int N>
__device__ __forceinline__ unsigned long long row16_min_u64_step(unsigned long long v) {
  const uint32_t oh = (uint32_t)row16_rot<N>((int)(uint32_t)(v >> 32)), ol = (uint32_t)row16_rot<N>((int)(uint32_t)v);
  const unsigned long long o = ((unsigned long long)oh << 32) | ol;
  return o < v ? o : v;
}
__device__ __forceinline__ unsigned long long grp32_min_u64(unsigned long long v) {
  v = row16_min_u64_step<8>(v); v = row16_min_u64_step<4>(v);
  v = row16_min_u64_step<2>(v); v = row16_min_u64_step<1>(v);
  const uint32_t oh = (uint32_t)swz_xor16((int)(uint32_t)(v >> 32)), ol = (uint32_t)swz_xor16((int)(uint32_t)v);
  const unsigned long long o = ((unsigned long long)oh << 32) | ol;
  return o < v ? o : v;
}
// Reductions over the LPS = 16 or 32 lanes that serve one slot
template <int LPS> __device__ __forceinline__ float grp_max(float v) { return LPS == 32 ? grp32_max(v) : row16_max(v); }
template <int LPS> __device__ __forceinline__ float grp_sum(float v) { return LPS == 32 ? grp32_sum(v) : row16_sum(v); }
template <int LPS> __device__ __forceinline__ int grp_sum(int v) { return LPS == 32 ? grp32_sum(v) : row16_sum(v); }
template <int LPS> __device__ __forceinline__ int grp_min(int v) { return LPS == 32 ? grp32_min(v) : row16_min(v); }
template <int LPS> __device__ __forceinline__ unsigned long long grp_min_u64(unsigned long long v) {
  if (LPS == 32) return grp32_min_u64(v);
  v = row16_min_u64_step<8>(v); v = row16_min_u64_step<4>(v);
  v = row16_min_u64_step<2>(v); v = row16_min_u64_step<1>(v);
  return v;
}
__device__ __forceinline__ void grp32_argmin(float& key, int& idx, float& payload) {
  row16_argmin(key, idx, payload);
  const float ok = swz_xor16(key), op = swz_xor16(payload);
  const int oi = swz_xor16(idx);
  if (ok < key || (ok == key && oi < idx)) { key = ok; idx = oi; payload = op; }
}

}  // namespace gfnx

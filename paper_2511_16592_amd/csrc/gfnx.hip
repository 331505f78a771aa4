// libgfnx_hip: C ABI (see include/gfnx.h), host-side validation, workspace layout and kernel launches.
#include "../../include/gfnx.h"

#include <hip/hip_runtime.h>

#include "gfnx_device.h"
#include "backward_kernel.h"
#include "grad_kernels.h"
#include "grad_kernels2.h"
#include "grad_kernels3.h"
#include "grad_kernels4.h"
#include "subtb_kernels.h"
#include "rollout_kernel.h"
#include "rollout_wide_kernel.h"

#include <cmath>
#include <mutex>
#include <string>
#include <vector>

using namespace gfnx;

namespace {

// ---- optional per-kernel timing (diagnostics): HIP events recorded on the launch stream around each kernel
struct TimingRecord { int label; hipEvent_t start, stop; };
bool g_timing_on = false;
std::string g_timing_only;  // when not empty, only this label is recorded
std::vector<std::string> g_labels;
std::vector<TimingRecord> g_records;
std::vector<hipEvent_t> g_event_pool;

int label_id(const char* name) {
  for (size_t i = 0; i < g_labels.size(); ++i) if (g_labels[i] == name) return (int)i;
  g_labels.push_back(name);
  return (int)g_labels.size() - 1;
}

hipEvent_t take_event() {
  if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

struct ScopedKernelTimer {
  hipStream_t st; int rec = -1;
  ScopedKernelTimer(const char* name, hipStream_t s) : st(s) {
    if (!g_timing_on) return;
    if (!g_timing_only.empty() && g_timing_only != name) return;
    TimingRecord r{label_id(name), take_event(), take_event()};
    (void)hipEventRecord(r.start, st);
    g_records.push_back(r);
    rec = (int)g_records.size() - 1;
  }
  ~ScopedKernelTimer() { if (rec >= 0) (void)hipEventRecord(g_records[rec].stop, st); }
};
#define GFNX_TIMED(name, stream) ScopedKernelTimer gfnx_timer_##__LINE__(name, stream)

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Shapes {
  int state_dim, obs_dim, n_actions, max_steps;
  int H1, H2, A, A16, B;
  size_t rows;  // max_steps * B
  int qt3, qtot3, s3, s2, qtot2;  // output tiling / split factors of dW3 and dW2
  int s1, qtot1;                  // ... of the one-hot dW1 contraction
  int mw1, mw2; // 64-bit sign-mask words per transition row for h1 / h2
  int flow;     // the network has one output more than the environment has actions: log F(s) (grids only)
  int onehot;   // layer-1 weight gradient as a one-hot contraction: 0 no, 1 grid, 2 Ising
  int sbytes;   // state bytes recorded per transition row for it
  int p1;       // rows of that contraction's output tile
  int wide;     // non-autoregressive bit sequences with more than 256 actions: 16-bit action plane, paged logits
};

struct Layout {
  size_t hdr, w2p, w3p, w3s, d1, crow, rows, h1, h2, e, lse, m1, m2, sb, part2, dbp2, part3, dbp3, part1, dbp1, cs;
  size_t phi, dl, lossb;  // flow networks: log F(s_t) and log P_F - log P_B per transition, loss per trajectory
  size_t total;
};

int env_dims(const gfnx_env_desc* env, int* sd, int* od, int* na, int* ms) {
  if (!env) return GFNX_E_NULL;
  if (env->kind == GFNX_ENV_GRID) {
    if (env->grid_dim < 1 || env->grid_dim > 16 || env->grid_side < 2 || env->grid_side > 127) return GFNX_E_BAD_ENV;
    *sd = env->grid_dim;
    *od = env->grid_dim * env->grid_side;
    *na = env->grid_dim + 1;
    *ms = env->grid_dim * (env->grid_side - 1) + 1;
  } else if (env->kind == GFNX_ENV_BITSEQ) {
    if (env->k_bits < 1 || env->k_bits > 8 || env->n_bits < env->k_bits || env->n_bits % env->k_bits) return GFNX_E_BAD_ENV;
    const int len = env->n_bits / env->k_bits;
    if (len > 32 || env->n_modes < 1) return GFNX_E_BAD_ENV;
    *sd = len;
    *od = len * ((1 << env->k_bits) + 1);
    *na = 1 << env->k_bits;
    *ms = len;
  } else if (env->kind == GFNX_ENV_ISING) {
    if (env->lattice_n < 3 || env->lattice_n > 10) return GFNX_E_BAD_ENV;
    const int d = env->lattice_n * env->lattice_n;
    *sd = d;
    *od = 3 * d;
    *na = 2 * d;
    *ms = d;
  } else if (env->kind == GFNX_ENV_BITSEQ_NA) {
    if (env->k_bits < 1 || env->k_bits > 8 || env->n_bits < env->k_bits || env->n_bits % env->k_bits) return GFNX_E_BAD_ENV;
    const int len = env->n_bits / env->k_bits;
    if (len > 32 || env->n_modes < 1) return GFNX_E_BAD_ENV;
    *sd = len;
    *od = len * ((1 << env->k_bits) + 1);
    *na = len << env->k_bits;
    *ms = len;
  } else {
    return GFNX_E_BAD_ENV;
  }
  return GFNX_OK;
}

int check_shapes(const gfnx_env_desc* env, const gfnx_mlp* mlp, int batch, Shapes* s) {
  if (!env || !mlp) return GFNX_E_NULL;
  int rc = env_dims(env, &s->state_dim, &s->obs_dim, &s->n_actions, &s->max_steps);
  if (rc) return rc;
  if ((env->kind == GFNX_ENV_BITSEQ || env->kind == GFNX_ENV_BITSEQ_NA) && !env->modes_dev) return GFNX_E_NULL;
  if (!mlp->W1 || !mlp->b1 || !mlp->W2 || !mlp->b2 || !mlp->W3 || !mlp->b3) return GFNX_E_NULL;
  if (batch <= 0) return GFNX_E_BAD_SHAPE;
  if (mlp->in_dim != s->obs_dim) return GFNX_E_BAD_SHAPE;
  s->flow = (env->kind == GFNX_ENV_GRID && mlp->n_actions == s->n_actions + 1) ? 1 : 0;
  if (!s->flow && mlp->n_actions != s->n_actions) return GFNX_E_BAD_SHAPE;
  if (mlp->h1 <= 0 || mlp->h2 <= 0) return GFNX_E_BAD_SHAPE;
  if (mlp->h1 % 64 || mlp->h2 % 64 || mlp->h1 > 512 || mlp->h2 > 512) return GFNX_E_UNSUPPORTED;
  // more than 256 actions: the non-autoregressive bit sequences only, in whole pages of 256 actions
  s->wide = s->n_actions > 256 ? 1 : 0;
  if (s->wide && (env->kind != GFNX_ENV_BITSEQ_NA || s->n_actions % 256 || s->n_actions > 8192)) return GFNX_E_UNSUPPORTED;
  if (s->max_steps > 256 || s->state_dim > kMaxStateDim) return GFNX_E_UNSUPPORTED;
  s->H1 = mlp->h1; s->H2 = mlp->h2; s->A = mlp->n_actions; s->A16 = (s->A + 15) & ~15; s->B = batch;
  s->rows = (size_t)s->max_steps * (size_t)batch;
  if (s->rows > 0x7fffffffull) return GFNX_E_UNSUPPORTED;
  s->mw1 = 4 * ((s->H1 + 255) / 256);
  s->mw2 = 4 * ((s->H2 + 255) / 256);
  s->onehot = 0; s->sbytes = 0; s->p1 = 0;
  if (env->kind == GFNX_ENV_GRID && s->obs_dim <= 256) { s->onehot = 1; s->sbytes = 16; s->p1 = s->obs_dim; }
  if (env->kind == GFNX_ENV_ISING) { s->onehot = 2; s->sbytes = 112; s->p1 = 2 * s->state_dim; }
  // Weight-gradient contractions: 256 x 256 output tiles (256 x 32 for at most 32 logits), the transitions split
  // over the workgroups so that about 256 of them run
  const int pt2 = (s->H1 + 255) / 256, qn2 = (s->H2 + 255) / 256, pt3 = (s->H2 + 255) / 256;
  s->qtot2 = 256 * qn2;
  s->s2 = 256 / (pt2 * qn2);
  s->qt3 = s->A16 <= 32 ? 32 : ((s->A16 > 192 && s->A16 <= 224) ? 224 : 256);  // 224: seven 32-column blocks per wave
  const int qn3 = s->A16 <= 256 ? 1 : (s->A16 + 255) / 256;
  s->qtot3 = s->qt3 * qn3;
  s->s3 = 256 / (pt3 * qn3) > 0 ? 256 / (pt3 * qn3) : 1;
  s->qtot1 = 256 * pt2;
  s->s1 = 256 / pt2;
  return GFNX_OK;
}

// Split parts of a weight-gradient contraction that can receive rows: a part holds at least three chunks of 32 rows
// (split_chunks_per_part), so small batches need far fewer partial tiles than the S workgroups launched.
inline size_t parts_in_use(const Shapes& s, int S) {
  const size_t chunks = (s.rows + 31) / 32, most = (chunks + 2) / 3;
  return most < (size_t)S ? (most ? most : 1) : (size_t)S;
}

Layout make_layout(const Shapes& s) {
  Layout L;
  size_t o = 0;
  L.hdr = o; o += align256(sizeof(int) * kHdrWords);
  L.w2p = o; o += align256(sizeof(float) * (size_t)s.H1 * s.H2);
  L.w3p = o; o += align256(sizeof(float) * (size_t)s.H2 * s.A16);
  // paged logit layer: W3 cut into bf16 pieces in the register order of the input-gradient kernel (6 bytes per weight)
  L.w3s = o; o += align256(s.wide ? (size_t)((s.H2 + 127) / 128) * 128 * s.A16 * 6 : 0);
  L.d1 = o; o += align256(s.wide ? 0 : sizeof(double) * (size_t)s.obs_dim * s.H1);  // difference rows of layer 1
  L.rows = o; o += align256(sizeof(int) * s.rows);
  L.crow = o; o += align256(sizeof(float) * s.rows);  // coefficient of each live transition
  L.h1 = o; o += align256(sizeof(float) * s.rows * s.H1);
  L.h2 = o; o += align256(sizeof(float) * s.rows * s.H2);
  L.e = o; o += align256(sizeof(float) * s.rows * s.A16);
  L.lse = o; o += align256(s.wide ? sizeof(float) * s.rows : 0);  // log-sum-exp of every row's valid logits
  L.m1 = o; o += align256(8 * s.rows * (size_t)s.mw1);
  L.m2 = o; o += align256(8 * s.rows * (size_t)s.mw2);
  L.sb = o; o += align256(s.rows * (size_t)s.sbytes);
  const size_t n1 = parts_in_use(s, s.s1), n2 = parts_in_use(s, s.s2), n3 = parts_in_use(s, s.s3);
  L.part1 = o; o += align256(s.onehot ? sizeof(float) * n1 * s.p1 * s.qtot1 : 0);
  L.dbp1 = o; o += align256(s.onehot ? sizeof(float) * n1 * s.qtot1 : 0);
  L.part2 = o; o += align256(sizeof(float) * n2 * s.H1 * s.qtot2);
  L.dbp2 = o; o += align256(sizeof(float) * n2 * s.qtot2);
  L.part3 = o; o += align256(sizeof(float) * n3 * s.H2 * s.qtot3);
  L.dbp3 = o; o += align256(sizeof(float) * n3 * s.qtot3);
  L.cs = o; o += align256(s.onehot ? 0 : sizeof(float) * (size_t)s.max_steps * s.H1);  // per-step column sums of G1
  L.phi = o; o += align256(s.flow ? sizeof(float) * s.rows : 0);
  L.dl = o; o += align256(s.flow ? sizeof(float) * s.rows : 0);
  L.lossb = o; o += align256(s.flow ? sizeof(float) * (size_t)(s.B + 2) : 0);
  L.total = o;
  return L;
}

int check_traj(const gfnx_traj* t, const Shapes& s) {
  if (!t) return GFNX_E_NULL;
  if (!(s.wide ? (const void*)t->actions16 : (const void*)t->actions)) return GFNX_E_NULL;
  if (!t->length || !t->terminal_state || !t->log_pf || !t->log_pb || !t->log_reward) return GFNX_E_NULL;
  if (t->batch <= 0 || t->max_steps < s.max_steps) return GFNX_E_BAD_SHAPE;
  return GFNX_OK;
}

int check_workspace(const void* ws, size_t bytes, const Layout& L) {
  if (!ws) return GFNX_E_WORKSPACE;
  if (((uintptr_t)ws) & 255) return GFNX_E_WORKSPACE;
  if (bytes < L.total) return GFNX_E_WORKSPACE;
  return GFNX_OK;
}

EnvParams env_params(const gfnx_env_desc* env, const Shapes& s) {
  EnvParams e = {};
  e.kind = env->kind;
  e.d = env->grid_dim; e.H = env->grid_side;
  e.r0 = env->r0; e.r1 = env->r1; e.r2 = env->r2;
  e.n_bits = env->n_bits; e.k_bits = env->k_bits; e.n_modes = env->n_modes;
  e.L = (env->kind == GFNX_ENV_BITSEQ || env->kind == GFNX_ENV_BITSEQ_NA) ? env->n_bits / env->k_bits : 0;
  e.words = (env->n_bits + 31) / 32;
  e.modes = env->modes_dev;
  e.beta = env->beta;
  e.N = env->lattice_n; e.D = env->lattice_n * env->lattice_n;
  e.coupling = env->coupling;
  e.state_dim = s.state_dim; e.obs_dim = s.obs_dim; e.n_actions = s.n_actions; e.max_steps = s.max_steps;
  return e;
}

template <typename T>
inline T* at(void* ws, size_t off) { return (T*)((char*)ws + off); }

// Workspace of the entry point that allocates nothing (gfnx_train_step_static): device memory that is part of the
// loaded code object, one copy per GPU at that GPU's own address.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the device address is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[GFNX_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GFNX_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return GFNX_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GFNX_OK;
}

// Raises a kernel's dynamic-LDS limit; the runtime call is made once per kernel instantiation and size (the
// largest size asked for so far is remembered per call site through `granted`).
template <typename K>
inline bool allow_lds(K kernel, int bytes, int* granted) {
  if (bytes <= *granted) return true;
  if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
  *granted = bytes;
  return true;
}
#define GFNX_ALLOW_LDS(kernel, bytes) \
  { static int granted_lds = 0; if (!allow_lds(kernel, (int)(bytes), &granted_lds)) return GFNX_E_HIP; }

// bytes per slot of the state kept in LDS by the rollout kernel
int rollout_state_pitch(const Shapes& s) {
  const int r = (s.state_dim + 15) / 16 * 16;
  return r > s.sbytes ? r : s.sbytes;
}

size_t rollout_lds_bytes(const Shapes& s, bool grid) {
  const bool stat = s.H1 == 256 && s.H2 == 256;
  return (size_t)rollout_lds_layout(s.H1, s.H2, s.A16, rollout_state_pitch(s), stat, grid && stat).total;
}

template <int ENV, bool REPLAY, int NCH, bool EXPLORE>
int launch_rollout_ntw(const RolloutParams& p, dim3 grid, size_t lds, hipStream_t st) {
#define GFNX_LAUNCH(N, STATIONARY, CA16)                                                                    \
  {                                                                                                         \
    auto k = rollout_kernel<ENV, REPLAY, N, STATIONARY, NCH, EXPLORE, CA16>;                                \
    GFNX_ALLOW_LDS(k, lds)                                                                                  \
    hipLaunchKernelGGL(k, grid, dim3(kRolloutThreads), lds, st, p);                                         \
  }
  if (p.H1 == 256 && p.H2 == 256) {  // layer 2 resident in registers
    // shapes of the benchmark configurations get the logit-tile shape as a compile-time constant
    if (ENV == 0 && p.A16 == 16) GFNX_LAUNCH(2, true, (ENV == 0 ? 16 : 0))
    else if (ENV == 2 && NCH == 2 && p.A16 == 208) GFNX_LAUNCH(2, true, (ENV == 2 && NCH == 2 ? 208 : 0))
    else GFNX_LAUNCH(2, true, 0)
    return GFNX_OK;
  }
  if (ENV == 1 && NCH == 2 && p.H2 == 512 && p.A16 == 256) {
    GFNX_LAUNCH(4, false, (ENV == 1 && NCH == 2 ? 256 : 0))
    return GFNX_OK;
  }
  switch ((p.H2 / 16 + 7) / 8) {  // 16-feature tiles of layer 2 per wave
    case 1: GFNX_LAUNCH(1, false, 0) break;
    case 2: GFNX_LAUNCH(2, false, 0) break;
    case 3: GFNX_LAUNCH(3, false, 0) break;
    case 4: GFNX_LAUNCH(4, false, 0) break;
    default: return GFNX_E_UNSUPPORTED;
  }
#undef GFNX_LAUNCH
  return GFNX_OK;
}

template <bool REPLAY, bool EXPLORE>
int launch_rollout(const RolloutParams& p, dim3 grid, size_t lds, hipStream_t st) {
  const bool wide = p.A16 > 128;  // more than one chunk of four logits per sampling lane
  switch (p.env.kind) {
    case GFNX_ENV_GRID: return launch_rollout_ntw<0, REPLAY, 1, EXPLORE>(p, grid, lds, st);
    case GFNX_ENV_BITSEQ:
      return wide ? launch_rollout_ntw<1, REPLAY, 2, EXPLORE>(p, grid, lds, st)
                  : launch_rollout_ntw<1, REPLAY, 1, EXPLORE>(p, grid, lds, st);
    case GFNX_ENV_BITSEQ_NA:
      return wide ? launch_rollout_ntw<3, REPLAY, 2, EXPLORE>(p, grid, lds, st)
                  : launch_rollout_ntw<3, REPLAY, 1, EXPLORE>(p, grid, lds, st);
    default:
      return wide ? launch_rollout_ntw<2, REPLAY, 2, EXPLORE>(p, grid, lds, st)
                  : launch_rollout_ntw<2, REPLAY, 1, EXPLORE>(p, grid, lds, st);
  }
}

int rollout_impl(const gfnx_env_desc* env, const gfnx_mlp* mlp, uint64_t seed, uint64_t iteration, gfnx_traj* traj,
                 void* ws, size_t ws_bytes, void* hip_stream, bool replay, float epsilon = 0.f) {
  Shapes s;
  if (!traj) return GFNX_E_NULL;
  if (!(epsilon >= 0.f && epsilon <= 1.f)) return GFNX_E_BAD_SHAPE;
  int rc = check_shapes(env, mlp, traj->batch, &s);
  if (rc) return rc;
  rc = check_traj(traj, s);
  if (rc) return rc;
  const Layout L = make_layout(s);
  rc = check_workspace(ws, ws_bytes, L);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;

  if (s.wide) {
    // more than 256 actions: the paged rollout of the non-autoregressive bit sequences
    WideParams q = {};
    q.eps = epsilon;
    q.env = env_params(env, s);
    q.In = s.obs_dim; q.H1 = s.H1; q.H2 = s.H2; q.A = s.A;
    q.W1 = mlp->W1; q.b1 = mlp->b1; q.b2 = mlp->b2; q.b3 = mlp->b3;
    q.W2p = at<float>(ws, L.w2p); q.W3p = at<float>(ws, L.w3p);
    q.seed_lo = (uint32_t)(seed & 0xFFFFFFFFull); q.seed_hi = (uint32_t)(seed >> 32);
    q.iter_lo = (uint32_t)(iteration & 0xFFFFFFFFull);
    q.B = s.B; q.T = traj->max_steps;
    q.actions = traj->actions16; q.length = traj->length; q.term = traj->terminal_state;
    q.lpf = traj->log_pf; q.lpb = traj->log_pb; q.logr = traj->log_reward;
    q.h1buf = at<float>(ws, L.h1); q.h2buf = at<float>(ws, L.h2); q.lgbuf = at<float>(ws, L.e);
    q.lsebuf = at<float>(ws, L.lse);
    q.m1buf = at<unsigned long long>(ws, L.m1); q.m2buf = at<unsigned long long>(ws, L.m2);
    q.MW1 = s.mw1; q.MW2 = s.mw2;
    int tpw = kSlots * ((s.B + 256 * kSlots - 1) / (256 * kSlots));
    q.tpw = tpw;
    const dim3 grid((s.B + tpw - 1) / tpw);
    const size_t lds = (size_t)wide_lds_layout(s.H1, s.H2).total;
    if (lds > 160 * 1024) return GFNX_E_UNSUPPORTED;
    {
      GFNX_TIMED("prepare", st);
      PrepareParams pp = {};
      pp.W1 = mlp->W1; pp.W2 = mlp->W2; pp.W3 = mlp->W3;
      pp.In = s.obs_dim; pp.H1 = s.H1; pp.H2 = s.H2; pp.A = s.A; pp.A16 = s.A16;
      pp.D1 = nullptr;  // layer 1 is summed from scratch every step
      pp.kind = (int)GFNX_ENV_BITSEQ; pp.group = (1 << env->k_bits) + 1;
      pp.W2p = at<float>(ws, L.w2p); pp.W3p = at<float>(ws, L.w3p);
      pp.actions = replay ? nullptr : (uint8_t*)traj->actions16;  // every 16-bit entry <- 0xFFFF
      pp.action_bytes = 2 * (size_t)traj->max_steps * s.B;
      hipLaunchKernelGGL(prepare_kernel, dim3(kPrepareBlocks), dim3(256), 0, st, pp);
    }
    {
      GFNX_TIMED("rollout", st);
      if (replay) {
        auto k = rollout_wide_kernel<true>;
        GFNX_ALLOW_LDS(k, (int)lds)
        hipLaunchKernelGGL(k, grid, dim3(kRolloutThreads), lds, st, q);
      } else {
        auto k = rollout_wide_kernel<false>;
        GFNX_ALLOW_LDS(k, (int)lds)
        hipLaunchKernelGGL(k, grid, dim3(kRolloutThreads), lds, st, q);
      }
    }
    return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
  }

  RolloutParams p = {};
  p.env = env_params(env, s);
  p.In = s.obs_dim; p.H1 = s.H1; p.H2 = s.H2; p.A = s.A; p.A16 = s.A16;
  p.W1 = mlp->W1; p.b1 = mlp->b1; p.b2 = mlp->b2; p.b3 = mlp->b3;
  p.W2p = at<float>(ws, L.w2p); p.W3p = at<float>(ws, L.w3p);
  p.D1 = at<double>(ws, L.d1);
  p.seed_lo = (uint32_t)(seed & 0xFFFFFFFFull); p.seed_hi = (uint32_t)(seed >> 32);
  p.iter_lo = (uint32_t)(iteration & 0xFFFFFFFFull);
  p.B = s.B; p.T = traj->max_steps;
  p.actions = traj->actions; p.length = traj->length; p.term = traj->terminal_state;
  p.lpf = traj->log_pf; p.lpb = traj->log_pb; p.logr = traj->log_reward;
  p.h1buf = at<float>(ws, L.h1); p.h2buf = at<float>(ws, L.h2); p.ebuf = at<float>(ws, L.e);
  p.m1buf = at<unsigned long long>(ws, L.m1);
  // sign masks of h2: read by the input-gradient GEMM of layer 3 only; the one-sweep logit backward of narrow action
  // spaces (same condition as in the gradient pass) takes the ReLU derivative from h2 itself
  p.m2buf = (s.A16 == 16 && s.H2 == 256) ? nullptr : at<unsigned long long>(ws, L.m2);
  p.MW1 = s.mw1; p.MW2 = s.mw2;
  p.sbuf = s.onehot ? at<uint8_t>(ws, L.sb) : nullptr;
  p.SB = s.sbytes;
  p.SBL = rollout_state_pitch(s);
  p.eps = epsilon;
  p.phibuf = s.flow ? at<float>(ws, L.phi) : nullptr;
  p.dlbuf = s.flow ? at<float>(ws, L.dl) : nullptr;

  // Each workgroup owns a contiguous range of trajectories and runs them 16 at a time; ranges longer than 16
  // (large batches) let a slot start the next trajectory as soon as its current one ends.
  int tpw = kSlots * ((s.B + 256 * kSlots - 1) / (256 * kSlots));
  if (tpw > 128) tpw = 128;
  p.tpw = tpw;
  const dim3 grid((s.B + tpw - 1) / tpw);
  const size_t lds = rollout_lds_bytes(s, env->kind == GFNX_ENV_GRID);
  if (lds > 160 * 1024) return GFNX_E_UNSUPPORTED;
  {
    // packed weights, difference rows, and (free-running rollout) every action byte preset to the 0xFF padding
    GFNX_TIMED("prepare", st);
    PrepareParams pp = {};
    pp.W1 = mlp->W1; pp.W2 = mlp->W2; pp.W3 = mlp->W3;
    pp.In = s.obs_dim; pp.H1 = s.H1; pp.H2 = s.H2; pp.A = s.A; pp.A16 = s.A16;
    pp.D1 = at<double>(ws, L.d1);
    pp.kind = env->kind == GFNX_ENV_BITSEQ_NA ? (int)GFNX_ENV_BITSEQ : env->kind;  // same "empty" row per position
    pp.group = env->kind == GFNX_ENV_GRID ? env->grid_side : (env->kind == GFNX_ENV_ISING ? 3 : (1 << env->k_bits) + 1);
    pp.W2p = at<float>(ws, L.w2p); pp.W3p = at<float>(ws, L.w3p);
    pp.actions = replay ? nullptr : traj->actions;
    pp.action_bytes = (size_t)traj->max_steps * s.B;
    hipLaunchKernelGGL(prepare_kernel, dim3(kPrepareBlocks), dim3(256), 0, st, pp);
  }
  {
    GFNX_TIMED("rollout", st);
    rc = replay ? launch_rollout<true, false>(p, grid, lds, st)
                : (epsilon > 0.f ? launch_rollout<false, true>(p, grid, lds, st)
                                 : launch_rollout<false, false>(p, grid, lds, st));
  }
  if (rc) return rc;
  return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
}

}  // namespace

extern "C" {

int gfnx_env_dims(const gfnx_env_desc* env, int32_t* state_dim, int32_t* obs_dim, int32_t* n_actions,
                  int32_t* max_steps) {
  int sd, od, na, ms;
  const int rc = env_dims(env, &sd, &od, &na, &ms);
  if (rc) return rc;
  if (state_dim) *state_dim = sd;
  if (obs_dim) *obs_dim = od;
  if (n_actions) *n_actions = na;
  if (max_steps) *max_steps = ms;
  return GFNX_OK;
}

size_t gfnx_workspace_bytes(const gfnx_env_desc* env, const gfnx_mlp* mlp, int32_t batch) {
  Shapes s;
  if (!env || !mlp) return 0;
  // size queries need the shapes only, not the device pointers
  gfnx_mlp m = *mlp;
  static const float dummy = 0.f;
  m.W1 = m.b1 = m.W2 = m.b2 = m.W3 = m.b3 = &dummy;
  gfnx_env_desc e = *env;
  if ((e.kind == GFNX_ENV_BITSEQ || e.kind == GFNX_ENV_BITSEQ_NA) && !e.modes_dev) e.modes_dev = (const uint32_t*)&dummy;
  if (check_shapes(&e, &m, batch, &s)) return 0;
  return make_layout(s).total;
}

int gfnx_workspace_region(const gfnx_env_desc* env, const gfnx_mlp* mlp, int32_t batch, int32_t region,
                          size_t* offset, size_t* row_bytes) {
  if (!env || !mlp || !offset || !row_bytes) return GFNX_E_NULL;
  Shapes s;
  gfnx_mlp m = *mlp;  // as in gfnx_workspace_bytes: the shapes only
  static const float dummy = 0.f;
  m.W1 = m.b1 = m.W2 = m.b2 = m.W3 = m.b3 = &dummy;
  gfnx_env_desc e = *env;
  if ((e.kind == GFNX_ENV_BITSEQ || e.kind == GFNX_ENV_BITSEQ_NA) && !e.modes_dev) e.modes_dev = (const uint32_t*)&dummy;
  const int rc = check_shapes(&e, &m, batch, &s);
  if (rc) return rc;
  const Layout L = make_layout(s);
  switch (region) {
    case GFNX_REGION_H1_SIGNS: *offset = L.m1; *row_bytes = 8 * (size_t)s.mw1; return GFNX_OK;
    case GFNX_REGION_H2_SIGNS:
      if (s.A16 == 16 && s.H2 == 256) return GFNX_E_UNSUPPORTED;  // not recorded: the gradient pass reads h2 itself
      *offset = L.m2; *row_bytes = 8 * (size_t)s.mw2; return GFNX_OK;
    case GFNX_REGION_H2_ROWS: *offset = L.h2; *row_bytes = sizeof(float) * (size_t)s.H2; return GFNX_OK;
    default: return GFNX_E_BAD_SHAPE;
  }
}

int gfnx_rollout(const gfnx_env_desc* env, const gfnx_mlp* mlp, uint64_t seed, uint64_t iteration, gfnx_traj* traj,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rollout_impl(env, mlp, seed, iteration, traj, workspace, workspace_bytes, hip_stream, false);
}

int gfnx_rollout_explore(const gfnx_env_desc* env, const gfnx_mlp* mlp, uint64_t seed, uint64_t iteration,
                         float epsilon, gfnx_traj* traj, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rollout_impl(env, mlp, seed, iteration, traj, workspace, workspace_bytes, hip_stream, false, epsilon);
}

int gfnx_replay(const gfnx_env_desc* env, const gfnx_mlp* mlp, gfnx_traj* traj, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  return rollout_impl(env, mlp, 0, 0, traj, workspace, workspace_bytes, hip_stream, true);
}

}  // extern "C"

namespace {

// log Z by value, or read from device memory when log_z_dev is not NULL
// With subtb_lambda >= 0: the Subtrajectory Balance objective of a network with a flow output instead of TB.
int tb_loss_grad_impl(const gfnx_env_desc* env, const gfnx_mlp* mlp, const gfnx_traj* traj, float log_z,
                      const float* log_z_dev, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads, void* ws,
                      size_t ws_bytes, void* hip_stream, float subtb_lambda = -1.f) {
  Shapes s;
  const bool subtb = subtb_lambda >= 0.f;
  if (!traj || !grads || !loss_dev || (!subtb && !dlogz_dev)) return GFNX_E_NULL;
  int rc = check_shapes(env, mlp, traj->batch, &s);
  if (rc) return rc;
  if (subtb != (s.flow != 0)) return GFNX_E_BAD_SHAPE;  // TB takes a plain policy network, SubTB one with a flow output
  rc = check_traj(traj, s);
  if (rc) return rc;
  if (!grads->dW1 || !grads->db1 || !grads->dW2 || !grads->db2 || !grads->dW3 || !grads->db3) return GFNX_E_NULL;
  const Layout L = make_layout(s);
  rc = check_workspace(ws, ws_bytes, L);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;

  int* hdr = at<int>(ws, L.hdr);
  int* rows = at<int>(ws, L.rows);
  float* crow = at<float>(ws, L.crow);
  float* h1buf = at<float>(ws, L.h1);
  float* h2buf = at<float>(ws, L.h2);
  float* ebuf = at<float>(ws, L.e);
  const int T = s.max_steps, B = s.B;
  if ((size_t)traj->max_steps * B > 0x7fffffffull) return GFNX_E_UNSUPPORTED;

  if (!subtb) {
    GFNX_TIMED("rows", st);
    hipLaunchKernelGGL(rows_kernel, dim3(T), dim3(1024), 0, st, traj->length, traj->log_pf, traj->log_pb, traj->log_reward,
                       log_z, log_z_dev, B, T, loss_dev, dlogz_dev, hdr, rows, crow);
  } else {
    // the same list of live rows (the TB scalars it also computes go to two scratch floats), then the per-transition
    // coefficients of the pair sum, which are folded into the logit-gradient rows so that every kernel below runs
    // unchanged with unit row coefficients
    float* lossb = at<float>(ws, L.lossb);
    float* phi = at<float>(ws, L.phi);
    float* dl = at<float>(ws, L.dl);
    GFNX_TIMED("rows", st);
    hipLaunchKernelGGL(rows_kernel, dim3(T), dim3(1024), 0, st, traj->length, traj->log_pf, traj->log_pb, traj->log_reward,
                       0.f, (const float*)nullptr, B, T, lossb + B, lossb + B + 1, hdr, rows, crow);
    hipLaunchKernelGGL(subtb_coef_kernel, dim3((B + 3) / 4), dim3(256), 0, st, (const int*)traj->length,
                       (const float*)traj->log_reward, phi, dl, B, T, subtb_lambda, lossb);
    hipLaunchKernelGGL(subtb_apply_kernel, dim3(512), dim3(256), 0, st, (const int*)rows, (const int*)hdr,
                       (const float*)dl, (const float*)phi, s.n_actions, s.A16, ebuf, crow, (const float*)lossb, B,
                       loss_dev);
  }
  if (s.wide) {
    // paged rollout: the stored logits of every live row become onehot(a) - p in place
    GFNX_TIMED("logit_grad", st);
    hipLaunchKernelGGL(wide_logit_grad_kernel, dim3(2048), dim3(256), 0, st, ebuf, (const float*)at<float>(ws, L.lse),
                       (const uint16_t*)traj->actions16, s.A, (const int*)rows, (const int*)hdr);
  }
  Dw1Params dp = {};
  dp.env = env_params(env, s);
  dp.H1 = s.H1; dp.B = B;
  dp.actions = traj->actions; dp.actions16 = s.wide ? traj->actions16 : nullptr; dp.length = traj->length; dp.term = traj->terminal_state;
  dp.g1 = h1buf; dp.dW1 = grads->dW1; dp.db1 = grads->db1;

  // the split partial tiles of every weight / bias gradient are summed by one launch at the end of the pass
  ReduceJobs jobs = {};
  auto add_job = [&](const float* part, int S, int P, int QTOT, int Q, float* out) {
    const int j = jobs.n++;
    jobs.part[j] = part; jobs.out[j] = out; jobs.S[j] = S; jobs.P[j] = P; jobs.QTOT[j] = QTOT; jobs.Q[j] = Q;
    jobs.first[j + 1] = jobs.first[j] + (P * (QTOT / 4) + 63) / 64;
  };
  float* part3 = at<float>(ws, L.part3);
  float* dbp3 = at<float>(ws, L.dbp3);
  float* part2 = at<float>(ws, L.part2);
  float* dbp2 = at<float>(ws, L.dbp2);
  const int pt2 = (s.H1 + 255) / 256, pt3 = (s.H2 + 255) / 256;
  // layer 3.  Narrow action spaces (at most 16 logits, 256 hidden units): dW3, db3 and G2 in one HBM-bound sweep
  // instead of two GEMMs that would be 16 wide
  const bool narrow = s.A16 == 16 && s.H2 == 256;
  if (narrow) {
    GFNX_TIMED("logit_bwd", st);
    auto k = logit_bwd_narrow_kernel;
    GFNX_ALLOW_LDS(k, kNarrowLdsBytes)
    hipLaunchKernelGGL(k, dim3(s.s3), dim3(512), kNarrowLdsBytes, st, h2buf, (const float*)ebuf, (const float*)crow,
                       mlp->W3, s.A, (const int*)rows, (const int*)hdr, part3, s.qtot3, dbp3);
  } else {
    // dW3 = H2^T G3, db3; G3 = coef * e is formed on load
    GFNX_TIMED("gemm_tn_w3", st);
    if (s.qt3 == 32) {
      auto k = gemm_tn3_kernel<8, 1, 1, 1, true>;
      const int lds = (int)gemm_tn3_lds_bytes<8, 1, 1, 1>();
      GFNX_ALLOW_LDS(k, lds)
      hipLaunchKernelGGL(k, dim3(pt3, 1, s.s3), dim3(512), lds, st, h2buf, s.H2, s.H2, ebuf, s.A16, (const float*)crow, rows, hdr,
                         s.qtot3, part3, dbp3);
    } else if (s.qt3 == 224) {
      // 193..224 logits (Ising 10 x 10: 200): a 256 x 224 tile, each wave 32 rows by seven column blocks, instead
      // of a 256 x 256 one an eighth of which would be padding
      auto k = gemm_tn3_kernel<8, 1, 1, 7, true>;
      const int lds = (int)gemm_tn3_lds_bytes<8, 1, 1, 7>();
      GFNX_ALLOW_LDS(k, lds)
      hipLaunchKernelGGL(k, dim3(pt3, 1, s.s3), dim3(512), lds, st, h2buf, s.H2, s.H2, ebuf, s.A16, (const float*)crow, rows, hdr,
                         s.qtot3, part3, dbp3);
    } else {
      auto k = gemm_tn3_kernel<2, 4, 4, 2, true>;
      const int lds = (int)gemm_tn3_lds_bytes<2, 4, 4, 2>();
      GFNX_ALLOW_LDS(k, lds)
      hipLaunchKernelGGL(k, dim3(pt3, s.qtot3 / 256, s.s3), dim3(512), lds, st, h2buf, s.H2, s.H2, ebuf, s.A16, (const float*)crow, rows, hdr,
                         s.qtot3, part3, dbp3);
    }
  }
  add_job(part3, s.s3, s.H2, s.qtot3, s.A, grads->dW3);
  add_job(dbp3, s.s3, 1, s.qtot3, s.A, grads->db3);
  const int rt32 = (int)((s.rows + kNt3Rows - 1) / kNt3Rows);
  // Out = (Gin W^T) . [act > 0] on the live rows, persistent over the row tiles: about one workgroup per CU
  auto launch_nt3 = [&](bool scale, const float* gin, int ldgi, int K, const float* W, int ldw, int kvalid, float* out,
                        int ldo, int P, const unsigned long long* mask, int mw) -> int {
#define GFNX_NT3(KH, SCALE, CTILES)                                                                               \
    {                                                                                                            \
      const int ctiles = (CTILES), lds = (int)gemm_nt3_lds_bytes<KH>();                                          \
      const int gx = rt32 < 256 / ctiles ? rt32 : (256 / ctiles > 0 ? 256 / ctiles : 1);                         \
      auto k = gemm_nt3_kernel<KH, SCALE>;                                                                       \
      GFNX_ALLOW_LDS(k, lds)                                                                                     \
      hipLaunchKernelGGL(k, dim3(gx, ctiles), dim3(512), lds, st, gin, ldgi, K, W, ldw, kvalid, out, ldo, P, mask, mw, \
                         (const float*)crow, (const int*)rows, (const int*)hdr);                                 \
    }
    if (K <= 256) {
      if (scale) GFNX_NT3(2, true, (P + 127) / 128)
      else GFNX_NT3(2, false, (P + 127) / 128)
    } else {
      // contraction lengths 257 .. 512: four contraction parts x two column blocks per workgroup (never scaled: only
      // layer 2 of a wide network is that long; the logit layer of the paged rollout has a kernel of its own)
      if (scale || K > 512) return GFNX_E_UNSUPPORTED;
      GFNX_NT3(4, false, (P + 63) / 64)
    }
#undef GFNX_NT3
    return GFNX_OK;
  };
  if (!narrow) {
    // G2 = ((coef * e) W3^T) . [h2 > 0] over h2
    GFNX_TIMED("gemm_nt_g2", st);
    if (!s.wide) {
      rc = launch_nt3(true, ebuf, s.A16, s.A16, mlp->W3, s.A, s.A, h2buf, s.H2, s.H2,
                      at<unsigned long long>(ws, L.m2), s.mw2);
      if (rc) return rc;
    } else {
      // the contraction over thousands of actions runs page by page (256 actions each, in order) inside one kernel,
      // against W3 cut into pieces beforehand
      const int pages = s.A / 256, ctiles = (s.H2 + 127) / 128;
      u32x4* w3s = at<u32x4>(ws, L.w3s);
      hipLaunchKernelGGL(split_w_pages_kernel, dim3(pages, ctiles), dim3(512), 0, st, mlp->W3, s.A, s.H2, pages, w3s);
      const int groups = (int)((s.rows + kNt3pTiles * kNt3Rows - 1) / (kNt3pTiles * kNt3Rows));
      const int per = 256 / ctiles >= 8 ? (256 / ctiles) & ~7 : 256 / ctiles;  // workers per column tile
      const int gx = groups < per ? groups : per;
      const int lds = (int)gemm_nt3p_lds_bytes();
      auto k = gemm_nt3p_kernel;
      GFNX_ALLOW_LDS(k, lds)
      hipLaunchKernelGGL(k, dim3(gx, ctiles), dim3(512), lds, st, (const float*)ebuf, s.A16, pages, (const u32x4*)w3s, h2buf,
                         s.H2, s.H2, (const unsigned long long*)at<unsigned long long>(ws, L.m2), s.mw2,
                         (const float*)crow, (const int*)rows, (const int*)hdr);
    }
  }
  {
    // layer 2: dW2 = H1^T G2, db2
    GFNX_TIMED("gemm_tn_w2", st);
    auto k = gemm_tn3_kernel<2, 4, 4, 2, false>;
    const int lds = (int)gemm_tn3_lds_bytes<2, 4, 4, 2>();
    GFNX_ALLOW_LDS(k, lds)
    hipLaunchKernelGGL(k, dim3(pt2, s.qtot2 / 256, s.s2), dim3(512), lds, st, h1buf, s.H1, s.H1, h2buf, s.H2, (const float*)crow, rows, hdr,
                       s.qtot2, part2, dbp2);
  }
  add_job(part2, s.s2, s.H1, s.qtot2, s.H2, grads->dW2);
  add_job(dbp2, s.s2, 1, s.qtot2, s.H2, grads->db2);
  {
    // G1 = (G2 W2^T) . [h1 > 0] over h1
    GFNX_TIMED("gemm_nt_g1", st);
    rc = launch_nt3(false, h2buf, s.H2, s.H2, mlp->W2, s.H2, s.H2, h1buf, s.H1, s.H1, at<unsigned long long>(ws, L.m1), s.mw1);
    if (rc) return rc;
  }
  // layer 1
  if (s.onehot) {
    // dW1 = onehot^T G1 on the matrix cores, the one-hot operand rebuilt from the recorded state bytes
    float* part1 = at<float>(ws, L.part1);
    float* dbp1 = at<float>(ws, L.dbp1);
    const uint8_t* sbuf = at<uint8_t>(ws, L.sb);
    const int lds = (int)dw1_onehot_lds_bytes();
    const dim3 grid1(s.s1, s.qtot1 / 256);
    {
      GFNX_TIMED("dw1", st);
      if (s.onehot == 1) {
        auto k = dw1_onehot_kernel<1>;
        GFNX_ALLOW_LDS(k, lds)
        hipLaunchKernelGGL(k, grid1, dim3(512), lds, st, (const float*)h1buf, s.H1, rows, hdr, sbuf, s.sbytes,
                           (int)env->grid_side, s.p1, s.qtot1, part1, dbp1);
      } else {
        auto k = dw1_onehot_kernel<2>;
        GFNX_ALLOW_LDS(k, lds)
        hipLaunchKernelGGL(k, grid1, dim3(512), lds, st, (const float*)h1buf, s.H1, rows, hdr, sbuf, s.sbytes, 1, s.p1,
                           s.qtot1, part1, dbp1);
      }
    }
    add_job(dbp1, s.s1, 1, s.qtot1, s.H1, grads->db1);
    if (s.onehot == 1) add_job(part1, s.s1, s.p1, s.qtot1, s.H1, grads->dW1);
  } else {
    // segment sums along each trajectory with atomics (large observation spaces: bit sequences)
    {
      GFNX_TIMED("fill_w1", st);
      hipLaunchKernelGGL(fill_kernel, dim3(512), dim3(256), 0, st, grads->dW1, (size_t)s.obs_dim * s.H1, 0.f);
      hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(256), 0, st, grads->db1, (size_t)s.H1, 0.f);
    }
    GFNX_TIMED("dw1", st);
    switch (env->kind) {
      case GFNX_ENV_GRID: hipLaunchKernelGGL(dw1_kernel<0>, dim3(B), dim3(256), 0, st, dp); break;
      case GFNX_ENV_BITSEQ: {
        // token rows: suffix sums per trajectory; the shared "empty" rows and db1: per-step column sums
        float* cs = at<float>(ws, L.cs);
        dp.suffix_only = 1;
        hipLaunchKernelGGL(fill_kernel, dim3(64), dim3(256), 0, st, cs, (size_t)T * s.H1, 0.f);
        hipLaunchKernelGGL(dw1_kernel<1>, dim3(B), dim3(256), 0, st, dp);
        hipLaunchKernelGGL(colsum_steps_kernel, dim3(T, 64), dim3(256), 0, st, (const float*)h1buf, s.H1, (const int*)rows,
                           (const int*)hdr, cs);
        hipLaunchKernelGGL(bitseq_empty_rows_kernel, dim3(s.state_dim), dim3(256), 0, st, (const float*)cs, s.H1,
                           s.state_dim, T, 1 << env->k_bits, grads->dW1, grads->db1);
        break;
      }
      case GFNX_ENV_BITSEQ_NA: {
        // token rows: suffix sums per trajectory; "empty" rows: the total (per-step column sums) minus the token rows
        float* cs = at<float>(ws, L.cs);
        dp.suffix_only = 1;
        hipLaunchKernelGGL(fill_kernel, dim3(64), dim3(256), 0, st, cs, (size_t)T * s.H1, 0.f);
        hipLaunchKernelGGL(dw1_kernel<3>, dim3(B), dim3(256), 0, st, dp);
        hipLaunchKernelGGL(colsum_steps_kernel, dim3(T, 64), dim3(256), 0, st, (const float*)h1buf, s.H1, (const int*)rows,
                           (const int*)hdr, cs);
        hipLaunchKernelGGL(na_empty_rows_kernel, dim3(s.state_dim, (s.H1 + 63) / 64), dim3(256), 0, st, (const float*)cs, s.H1, T,
                           1 << env->k_bits, grads->dW1, grads->db1);
        break;
      }
      default: hipLaunchKernelGGL(dw1_kernel<2>, dim3(B), dim3(256), 0, st, dp); break;
    }
  }
  {
    GFNX_TIMED("reduce", st);
    hipLaunchKernelGGL(reduce_jobs_kernel, dim3(jobs.first[jobs.n]), dim3(256), 0, st, jobs, (const int*)hdr);
    if (s.onehot == 2)  // needs db1 from the launch above
      hipLaunchKernelGGL(reduce_dw1_ising_kernel, dim3((s.p1 / 2 * (s.H1 / 4) + 63) / 64), dim3(256), 0, st,
                         (const float*)at<float>(ws, L.part1), s.s1, s.p1, s.qtot1, s.H1, (const int*)hdr, grads->db1, grads->dW1);
  }
  return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
}

int check_adam(const gfnx_mlp* mlp, float* log_z_dev, const gfnx_mlp_grad* grads, const float* dlogz_dev,
               const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step) {
  if (!mlp || !grads || !state || !cfg) return GFNX_E_NULL;
  if (!mlp->W1 || !mlp->b1 || !mlp->W2 || !mlp->b2 || !mlp->W3 || !mlp->b3) return GFNX_E_NULL;
  if (!grads->dW1 || !grads->db1 || !grads->dW2 || !grads->db2 || !grads->dW3 || !grads->db3) return GFNX_E_NULL;
  for (const gfnx_mlp_grad* q : {&state->m, &state->v})
    if (!q->dW1 || !q->db1 || !q->dW2 || !q->db2 || !q->dW3 || !q->db3) return GFNX_E_NULL;
  const int nz = (log_z_dev != nullptr) + (dlogz_dev != nullptr) + (state->log_z_mv != nullptr);
  if (nz != 0 && nz != 3) return GFNX_E_NULL;
  if (mlp->in_dim <= 0 || mlp->h1 <= 0 || mlp->h2 <= 0 || mlp->n_actions <= 0) return GFNX_E_BAD_SHAPE;
  if ((uint64_t)mlp->in_dim * mlp->h1 > 0x7fffffffull || (uint64_t)mlp->h1 * mlp->h2 > 0x7fffffffull ||
      (uint64_t)mlp->h2 * mlp->n_actions > 0x7fffffffull)
    return GFNX_E_UNSUPPORTED;
  if (step < 1) return GFNX_E_BAD_SHAPE;
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f)) return GFNX_E_BAD_SHAPE;
  if (!(cfg->lr >= 0.f) || !(cfg->lr_log_z >= 0.f) || !(cfg->eps >= 0.f)) return GFNX_E_BAD_SHAPE;
  return GFNX_OK;
}

int adam_impl(const gfnx_mlp* mlp, float* log_z_dev, const gfnx_mlp_grad* grads, const float* dlogz_dev,
              const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* hip_stream) {
  const int rc = check_adam(mlp, log_z_dev, grads, dlogz_dev, state, cfg, step);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  AdamJobs a = {};
  auto add = [&](const float* theta, const float* g, float* m, float* v, size_t n, float lr) {
    const int j = a.jobs++;
    a.theta[j] = const_cast<float*>(theta); a.g[j] = g; a.m[j] = m; a.v[j] = v; a.n[j] = (unsigned)n; a.lr[j] = lr;
    a.first[j + 1] = a.first[j] + (int)((n + 1023) / 1024);
  };
  const size_t In = mlp->in_dim, H1 = mlp->h1, H2 = mlp->h2, A = mlp->n_actions;
  add(mlp->W1, grads->dW1, state->m.dW1, state->v.dW1, In * H1, cfg->lr);
  add(mlp->b1, grads->db1, state->m.db1, state->v.db1, H1, cfg->lr);
  add(mlp->W2, grads->dW2, state->m.dW2, state->v.dW2, H1 * H2, cfg->lr);
  add(mlp->b2, grads->db2, state->m.db2, state->v.db2, H2, cfg->lr);
  add(mlp->W3, grads->dW3, state->m.dW3, state->v.dW3, H2 * A, cfg->lr);
  add(mlp->b3, grads->db3, state->m.db3, state->v.db3, A, cfg->lr);
  if (log_z_dev) add(log_z_dev, dlogz_dev, state->log_z_mv, state->log_z_mv + 1, 1, cfg->lr_log_z);
  a.beta1 = cfg->beta1; a.beta2 = cfg->beta2; a.eps = cfg->eps;
  a.c1 = 1.f - (float)pow((double)cfg->beta1, (double)step);
  a.c2 = 1.f - (float)pow((double)cfg->beta2, (double)step);
  {
    GFNX_TIMED("adam", st);
    hipLaunchKernelGGL(adam_kernel, dim3(a.first[a.jobs]), dim3(256), 0, st, a);
  }
  return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
}

}  // namespace

extern "C" {

int gfnx_tb_loss_grad(const gfnx_env_desc* env, const gfnx_mlp* mlp, const gfnx_traj* traj, float log_z,
                      float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads, void* ws, size_t ws_bytes,
                      void* hip_stream) {
  return tb_loss_grad_impl(env, mlp, traj, log_z, nullptr, loss_dev, dlogz_dev, grads, ws, ws_bytes, hip_stream);
}

int gfnx_subtb_loss_grad(const gfnx_env_desc* env, const gfnx_mlp* mlp, const gfnx_traj* traj, float lambda,
                         float* loss_dev, gfnx_mlp_grad* grads, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!(lambda >= 0.f && lambda <= 1.f)) return GFNX_E_BAD_SHAPE;
  return tb_loss_grad_impl(env, mlp, traj, 0.f, nullptr, loss_dev, nullptr, grads, ws, ws_bytes, hip_stream, lambda);
}

int gfnx_backward_rollout(const gfnx_env_desc* env, uint64_t seed, uint64_t iteration, gfnx_traj* traj,
                          void* hip_stream) {
  if (!env || !traj) return GFNX_E_NULL;
  int sd, od, na, ms;
  const int rc = env_dims(env, &sd, &od, &na, &ms);
  if (rc) return rc;
  const bool wide = na > 256;  // 16-bit action plane (non-autoregressive bit sequences only)
  if (!(wide ? (const void*)traj->actions16 : (const void*)traj->actions)) return GFNX_E_NULL;
  if (!traj->length || !traj->terminal_state || !traj->log_pb) return GFNX_E_NULL;
  if (traj->batch <= 0 || traj->max_steps < ms) return GFNX_E_BAD_SHAPE;
  if ((wide && (env->kind != GFNX_ENV_BITSEQ_NA || na % 256 || na > 8192)) || ms > 256 || sd > kMaxStateDim)
    return GFNX_E_UNSUPPORTED;  // the limits of the forward kernels
  if (env->kind == GFNX_ENV_GRID && sd > 16) return GFNX_E_UNSUPPORTED;
  if ((size_t)traj->max_steps * (size_t)traj->batch > 0x7fffffffull) return GFNX_E_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  BackwardParams p = {};
  Shapes s = {};
  s.state_dim = sd; s.obs_dim = od; s.n_actions = na; s.max_steps = ms;
  p.env = env_params(env, s);
  p.seed_lo = (uint32_t)(seed & 0xFFFFFFFFull); p.seed_hi = (uint32_t)(seed >> 32);
  p.iter_lo = (uint32_t)(iteration & 0xFFFFFFFFull);
  p.B = traj->batch; p.T = traj->max_steps;
  p.term = traj->terminal_state; p.actions = traj->actions; p.actions16 = wide ? traj->actions16 : nullptr;
  p.length = traj->length; p.lpb = traj->log_pb;
  {
    GFNX_TIMED("backward", st);
    hipLaunchKernelGGL(backward_rollout_kernel, dim3((p.B + kBackwardThreads - 1) / kBackwardThreads),
                       dim3(kBackwardThreads), 0, st, p);
  }
  return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
}

int gfnx_log_prob_estimate(const float* log_pf_dev, const float* log_pb_dev, int32_t n_states, int32_t n_samples,
                           float* log_p_dev, void* hip_stream) {
  if (!log_pf_dev || !log_pb_dev || !log_p_dev) return GFNX_E_NULL;
  if (n_states < 1 || n_samples < 1) return GFNX_E_BAD_SHAPE;
  if ((uint64_t)n_states * (uint64_t)n_samples > 0x7fffffffull) return GFNX_E_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  {
    GFNX_TIMED("estimate", st);
    hipLaunchKernelGGL(log_prob_estimate_kernel, dim3((n_states + 3) / 4), dim3(256), 0, st, log_pf_dev, log_pb_dev,
                       n_states, n_samples, log_p_dev);
  }
  return hipGetLastError() == hipSuccess ? GFNX_OK : GFNX_E_HIP;
}

int gfnx_adam_step(const gfnx_mlp* mlp, float* log_z_dev, const gfnx_mlp_grad* grads, const float* dlogz_dev,
                   const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* hip_stream) {
  return adam_impl(mlp, log_z_dev, grads, dlogz_dev, state, cfg, step, hip_stream);
}

int gfnx_train_step_opts(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                         uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                         const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, const gfnx_train_opts* opts,
                         int64_t step, void* ws, size_t ws_bytes, void* hip_stream) {
  // every argument is checked before the first launch, so a rejected call leaves all buffers untouched
  if (!opts || !loss_dev || !grads || !traj || !state) return GFNX_E_NULL;
  if (!(opts->epsilon >= 0.f && opts->epsilon <= 1.f)) return GFNX_E_BAD_SHAPE;
  const bool subtb = opts->subtb_lambda >= 0.f;
  if (subtb && !(opts->subtb_lambda <= 1.f)) return GFNX_E_BAD_SHAPE;
  if (!subtb && !(opts->subtb_lambda < 0.f)) return GFNX_E_BAD_SHAPE;  // NaN
  gfnx_adam_state st = *state;
  if (subtb) {  // no log Z in this objective: the flow output at s_0 plays its part
    log_z_dev = nullptr;
    dlogz_dev = nullptr;
    st.log_z_mv = nullptr;
  } else if (!log_z_dev || !dlogz_dev) {
    return GFNX_E_NULL;
  }
  int rc = check_adam(mlp, log_z_dev, grads, dlogz_dev, &st, cfg, step);
  if (rc) return rc;
  {
    Shapes s;
    rc = check_shapes(env, mlp, traj->batch, &s);
    if (rc) return rc;
    if (subtb != (s.flow != 0)) return GFNX_E_BAD_SHAPE;  // TB: plain policy network; SubTB: one with a flow output
  }
  rc = rollout_impl(env, mlp, seed, iteration, traj, ws, ws_bytes, hip_stream, false, opts->epsilon);
  if (rc) return rc;
  rc = tb_loss_grad_impl(env, mlp, traj, 0.f, log_z_dev, loss_dev, dlogz_dev, grads, ws, ws_bytes, hip_stream,
                         subtb ? opts->subtb_lambda : -1.f);
  if (rc) return rc;
  return adam_impl(mlp, log_z_dev, grads, dlogz_dev, &st, cfg, step, hip_stream);
}

int gfnx_train_step(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                    uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                    const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* ws, size_t ws_bytes,
                    void* hip_stream) {
  const gfnx_train_opts opts = {0.f, -1.f};
  return gfnx_train_step_opts(env, mlp, log_z_dev, seed, iteration, traj, loss_dev, dlogz_dev, grads, state, cfg, &opts,
                              step, ws, ws_bytes, hip_stream);
}

int gfnx_train_step_static(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                           uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                           const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* hip_stream) {
  // the size is checked on the host before the runtime is touched
  if (!env || !mlp || !traj) return GFNX_E_NULL;
  const size_t need = gfnx_workspace_bytes(env, mlp, traj->batch);
  if (need == 0) {  // let the shape checks name the error
    Shapes s;
    const int rc = check_shapes(env, mlp, traj->batch, &s);
    return rc ? rc : GFNX_E_BAD_SHAPE;
  }
  if (need > (size_t)GFNX_STATIC_SCRATCH_BYTES) return GFNX_E_WORKSPACE;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc) return rc;
  return gfnx_train_step(env, mlp, log_z_dev, seed, iteration, traj, loss_dev, dlogz_dev, grads, state, cfg, step, ws,
                         (size_t)GFNX_STATIC_SCRATCH_BYTES, hip_stream);
}

int gfnx_timing_enable(int on) {
  for (auto& r : g_records) { g_event_pool.push_back(r.start); g_event_pool.push_back(r.stop); }
  g_records.clear();
  g_timing_on = on != 0;
  return GFNX_OK;
}

int gfnx_timing_only(const char* label) {
  g_timing_only = label ? label : "";
  return GFNX_OK;
}

int gfnx_timing_labels(void) { return (int)g_labels.size(); }

int gfnx_timing_get(int label, const char** name, int32_t* launches, float* total_ms) {
  if (label < 0 || label >= (int)g_labels.size() || !name || !launches || !total_ms) return GFNX_E_NULL;
  *name = g_labels[label].c_str();
  *launches = 0;
  *total_ms = 0.f;
  for (auto& r : g_records) {
    if (r.label != label) continue;
    if (hipEventSynchronize(r.stop) != hipSuccess) return GFNX_E_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return GFNX_E_HIP;
    *launches += 1;
    *total_ms += ms;
  }
  return GFNX_OK;
}

const char* gfnx_status_string(int status) {
  switch (status) {
    case GFNX_OK: return "GFNX_OK";
    case GFNX_E_NULL: return "GFNX_E_NULL: a required pointer is NULL";
    case GFNX_E_BAD_ENV: return "GFNX_E_BAD_ENV: inconsistent environment descriptor";
    case GFNX_E_BAD_SHAPE: return "GFNX_E_BAD_SHAPE: shapes do not match the environment";
    case GFNX_E_WORKSPACE: return "GFNX_E_WORKSPACE: workspace missing, misaligned or too small";
    case GFNX_E_UNSUPPORTED: return "GFNX_E_UNSUPPORTED: outside the supported sizes";
    case GFNX_E_HIP: return "GFNX_E_HIP: HIP runtime error";
    default: return "unknown gfnx status";
  }
}

}  // extern "C"

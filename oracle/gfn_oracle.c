/*
 * gfn_oracle.c -- plain CPU reference ("oracle") for the GFlowNet rollout +
 * Trajectory-Balance gradient path.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow on purpose, shares no code with the
 * GPU library, and must only be used by the tests, by the smoke check and by the
 * CPU-baseline leg of the benchmark.  Nothing in the product path may call it.
 *
 * The file is compiled twice: -DORACLE_REAL=float gives liboracle_f32.so (all
 * arithmetic in binary32, used where a floating-point comparison decides an
 * integer: the sampled action), -DORACLE_REAL=double gives liboracle_f64.so
 * (used as the ground truth for log-probabilities, the loss and the gradients
 * along a given action sequence, and for finite differences).
 *
 * What is computed, with the passage of the paper each part follows:
 *   - trajectories and the forward / backward trajectory distributions:
 *     Background section, eq. (tb) and eq. (forward_backward_traj);
 *   - Trajectory Balance objective: Background section, eq. (TB_loss), with a
 *     fixed uniform backward policy (last paragraph of that section);
 *   - hypergrid environment and reward: Appendix "Hypergrid", reward equation,
 *     and the usage listing in "Library Details" (stop action is the LAST index);
 *   - bit sequences, autoregressive fixed-length scheme: Appendix "Sequential
 *     environments" (generation schemes) and "Bit sequences" (reward equation); and in the
 *     non-autoregressive scheme of the same appendix, the one the paper's bit-sequence
 *     experiments use (an action = an empty position and the k-bit word written there;
 *     backward actions remove the word of any filled position);
 *   - Ising partial assignments: Appendix "Ising model" (energy equation,
 *     state / action description);
 *   - environments emit log-reward only on the terminal transition: "Library
 *     Details", implementation notes;
 *   - Detailed Balance and Subtrajectory Balance objectives with a learned state flow: Background section,
 *     eq. (DB_loss) and eq. (SubTB_loss) (weights lambda^(k-j) normalised to sum to one, flow of a terminal
 *     state replaced by its reward);
 *   - backward rollouts and the Monte-Carlo estimate of the probability P_theta(x) of
 *     sampling a terminal state x: "Library Details" (a backward rollout is a rollout
 *     started at terminal states with the backward step in place of the step; backward
 *     actions are the structural choices only) and Appendix "Bit sequences" (estimator
 *     equation: mean over tau^i ~ P_B(.|x) of P_F(tau^i) / P_B(tau^i | x));
 *   - the optimiser step of a training iteration: Adam with the settings of the
 *     hypergrid hyperparameter table (Appendix "Hypergrid": learning rate 1e-3,
 *     1e-1 for log Z, betas (0.9, 0.999), epsilon 1e-8, no weight decay), the
 *     update itself as published by Kingma & Ba (2015), Algorithm 1.
 *
 * Conventions fixed here where the paper is silent (they are listed in full in
 * the design document of the repository):
 *   MLP      y = b + sum_i x_i W[i][:], W row-major [in][out], ReLU on both hidden
 *            layers, ReLU'(0) = 0, sums taken in increasing index order starting
 *            from the bias.
 *   one-hot  grid: index H*i + x_i;  bitseq: 257*pos + tok (tok 256 = empty);
 *            Ising: 3*site + (x+1) with x in {-1, 0(unassigned), +1}.
 *   actions  grid: a<d increments coordinate a, a==d stops;  bitseq: step t writes
 *            token a at position t;  Ising: site = a/2, spin = 2*(a%2)-1;  non-autoregressive
 *            bitseq: position = a / 2^k, word = a % 2^k, valid iff the position is empty.
 *   sampler  Gumbel-max over the valid actions, lowest index wins exact ties.
 *   RNG      Philox4x32-10 (Salmon et al., SC'11): key = (seed lo, seed hi),
 *            counter = (trajectory b, step t, a/4, iteration lo); output word a%4
 *            serves action a.  u = ((w>>9)+0.5)*2^-23,  g = -log(-log(u)).
 *   log P_B  grid increment: -log #{i : child_i > 0}; grid stop: 0; bitseq: 0;
 *            Ising: -log(#assigned sites of the child) = -log(t+1); non-autoregressive bitseq:
 *            -log(#filled positions of the child) = -log(t+1).
 *   explore  epsilon-uniform exploration: one more Philox call per step, counter (b, t,
 *            0xFFFFFFFE, iteration lo); word 0 -> u, explore iff u < epsilon (binary32);
 *            word 1 -> the j-th valid action in increasing order, j = floor(w * n / 2^32).
 *   backward the parents of a state in increasing index order (grid: coordinates > 0;
 *            Ising: assigned sites; bitseq: the last position only); the j-th is taken,
 *            j = floor(w * n / 2^32), w = word 0 of Philox(counter = (b, k, 0xFFFFFFFF,
 *            iteration lo)), k = index of the backward move (the grid's un-stop move has
 *            one parent and draws nothing).
 *   loss     mean over the batch of the squared residual
 *            delta_b = log Z + log P_F(tau_b) - log R(x_b) - log P_B(tau_b).
 *
 * Parity pins (tests/test_oracle_*.py): exhaustive enumeration on the 2-D side-4
 * grid, closed-form normalising constants, the DP-optimal policy with zero
 * residual, closed-form rewards, finite differences, an independent big-integer
 * Philox and the published known-answer vectors, chi-square tests of the sampler;
 * for the optimiser step a library Adam, the constant-gradient closed form, and a
 * training run on the side-4 grid whose terminal distribution must approach R/Z;
 * for backward rollouts reversibility, path frequencies against the enumeration and
 * the estimate being exactly R(x)/Z under the proper policy; for exploration the
 * uniform and mixture frequencies; for DB / SubTB zero loss under the proper policy
 * with the true state flows, the pair sum written out, and finite differences.
 * Free-running sampled actions have no external reference ("parity unpinned"
 * beyond those statistical pins): the counter layout above is this implementation's own.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

#define ENV_GRID 0
#define ENV_BITSEQ 1
#define ENV_ISING 2
#define ENV_BITSEQ_NA 3 /* bit sequences, non-autoregressive scheme: an action picks an empty position and a word */

#define MAX_STATE 1024
#define MAX_ACT 4096
/* One action per (step, trajectory) in 16 bits (the non-autoregressive bit sequences of the paper's experiments have
 * 15 x 256 = 3840 actions); ACT_PAD fills the steps past the end of a trajectory. */
typedef uint16_t act_t;
#define ACT_PAD 0xFFFFu

typedef struct {
  int32_t kind;
  int32_t grid_dim, grid_side;
  double r0, r1, r2;
  int32_t n_bits, k_bits, n_modes;
  const uint32_t* modes; /* n_modes x ceil(n_bits/32) words, host */
  double beta;
  int32_t lattice_n;
  double coupling;
} oracle_env;

typedef struct {
  int32_t in_dim, h1, h2, n_actions;
  const real *W1, *b1, *W2, *b2, *W3, *b3;
} oracle_mlp;

typedef struct {
  real *dW1, *db1, *dW2, *db2, *dW3, *db3;
} oracle_grad;

/* ------------------------------------------------------------------ RNG */

static uint32_t mulhi32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32); }

/* Philox4x32 with 10 rounds, as defined by Salmon, Moraes, Dror and Shaw,
 * "Parallel random numbers: as easy as 1, 2, 3" (SC'11). */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 32 random bits -> uniform strictly inside (0,1), exactly representable in binary32. */
real oracle_uniform(uint32_t w) { return ((real)(w >> 9) + (real)0.5) * (real)(1.0 / 8388608.0); }

static real rlog(real x) { return sizeof(real) == 4 ? (real)logf((float)x) : (real)log((double)x); }
static real rexp(real x) { return sizeof(real) == 4 ? (real)expf((float)x) : (real)exp((double)x); }
static real rabs(real x) { return x < 0 ? -x : x; }

real oracle_gumbel(uint32_t w) { return -rlog(-rlog(oracle_uniform(w))); }

static real action_noise(uint64_t seed, uint64_t iteration, uint32_t b, uint32_t t, int a) {
  uint32_t ctr[4] = {b, t, (uint32_t)(a / 4), (uint32_t)(iteration & 0xFFFFFFFFu)};
  uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  return oracle_gumbel(out[a % 4]);
}

/* ------------------------------------------------------------ environments */

int oracle_env_dims(const oracle_env* e, int32_t* state_dim, int32_t* obs_dim, int32_t* n_actions, int32_t* max_steps) {
  if (e->kind == ENV_GRID) {
    *state_dim = e->grid_dim;
    *obs_dim = e->grid_dim * e->grid_side;
    *n_actions = e->grid_dim + 1;
    *max_steps = e->grid_dim * (e->grid_side - 1) + 1;
  } else if (e->kind == ENV_BITSEQ) {
    int len = e->n_bits / e->k_bits;
    *state_dim = len;
    *obs_dim = len * ((1 << e->k_bits) + 1);
    *n_actions = 1 << e->k_bits;
    *max_steps = len;
  } else if (e->kind == ENV_ISING) {
    int d = e->lattice_n * e->lattice_n;
    *state_dim = d;
    *obs_dim = 3 * d;
    *n_actions = 2 * d;
    *max_steps = d;
  } else if (e->kind == ENV_BITSEQ_NA) {
    int len = e->n_bits / e->k_bits;
    *state_dim = len;
    *obs_dim = len * ((1 << e->k_bits) + 1);
    *n_actions = len << e->k_bits;
    *max_steps = len;
  } else {
    return -1;
  }
  return 0;
}

/* state vector s[state_dim]: grid coordinate; bitseq token (empty = 2^k); Ising spin (0 = unassigned) */
static void env_reset(const oracle_env* e, int* s, int sd) {
  for (int i = 0; i < sd; ++i) s[i] = (e->kind == ENV_BITSEQ || e->kind == ENV_BITSEQ_NA) ? (1 << e->k_bits) : 0;
}

/* indices of the non-zero entries of the one-hot observation, in increasing order */
static int env_obs_rows(const oracle_env* e, const int* s, int sd, int* rows) {
  for (int i = 0; i < sd; ++i) {
    if (e->kind == ENV_GRID) rows[i] = e->grid_side * i + s[i];
    else if (e->kind == ENV_BITSEQ || e->kind == ENV_BITSEQ_NA) rows[i] = ((1 << e->k_bits) + 1) * i + s[i];
    else rows[i] = 3 * i + (s[i] + 1);
  }
  return sd;
}

static void env_valid(const oracle_env* e, const int* s, int t, int n_actions, int* valid) {
  (void)t;
  for (int a = 0; a < n_actions; ++a) {
    if (e->kind == ENV_GRID) valid[a] = (a == e->grid_dim) ? 1 : (s[a] < e->grid_side - 1);
    else if (e->kind == ENV_BITSEQ) valid[a] = 1;
    else if (e->kind == ENV_BITSEQ_NA) valid[a] = (s[a >> e->k_bits] == (1 << e->k_bits));
    else valid[a] = (s[a / 2] == 0);
  }
}

/* applies action a at step t; returns 1 if the child is terminal */
static int env_step(const oracle_env* e, int* s, int sd, int t, int a) {
  if (e->kind == ENV_GRID) {
    if (a == e->grid_dim) return 1; /* the terminal copy keeps the coordinates */
    s[a] += 1;
    return 0;
  }
  if (e->kind == ENV_BITSEQ) {
    s[t] = a;
    return t + 1 == sd;
  }
  if (e->kind == ENV_BITSEQ_NA) {
    s[a >> e->k_bits] = a & ((1 << e->k_bits) - 1);
    return t + 1 == sd; /* every step fills one position: terminal when none is empty */
  }
  s[a / 2] = 2 * (a % 2) - 1;
  return t + 1 == sd;
}

/* log P_B(parent | child) under the uniform backward policy; s is the CHILD state */
static real env_log_pb(const oracle_env* e, const int* s, int sd, int t, int a) {
  if (e->kind == ENV_GRID) {
    if (a == e->grid_dim) return 0;
    int count = 0;
    for (int i = 0; i < sd; ++i) count += (s[i] > 0);
    return -rlog((real)count);
  }
  if (e->kind == ENV_BITSEQ) return 0;
  return -rlog((real)(t + 1)); /* Ising, non-autoregressive bitseq: the child has t+1 assigned sites / filled positions */
}

static real env_log_reward(const oracle_env* e, const int* s, int sd) {
  if (e->kind == ENV_GRID) {
    /* The indicators of the reward equation compare v = |x / (H-1) - 1/2| with 1/4, 3/10 and 2/5, strictly.  A
     * coordinate can sit exactly on a threshold (H-1 a multiple of 4, 5 or 10), so the comparisons are made on
     * integers, where they are exact:  1/4 < v  <=>  H-1 < |4x - 2(H-1)|;   3/10 < v < 2/5  <=>
     * 3(H-1) < |10x - 5(H-1)| < 4(H-1). */
    int in1 = 1, in2 = 1;
    const int h = e->grid_side - 1;
    for (int i = 0; i < sd; ++i) {
      const int q = abs(4 * s[i] - 2 * h), r = abs(10 * s[i] - 5 * h);
      in1 = in1 && (h < q);
      in2 = in2 && (3 * h < r) && (r < 4 * h);
    }
    real r = (real)e->r0 + (real)e->r1 * (real)in1 + (real)e->r2 * (real)in2;
    return rlog(r);
  }
  if (e->kind == ENV_BITSEQ || e->kind == ENV_BITSEQ_NA) {
    int k = e->k_bits, n = e->n_bits, words = (n + 31) / 32;
    int dmin = n + 1;
    for (int m = 0; m < e->n_modes; ++m) {
      int dist = 0;
      for (int i = 0; i < n; ++i) {
        int xbit = (s[i / k] >> (k - 1 - i % k)) & 1;
        int mbit = (int)((e->modes[(size_t)m * words + i / 32] >> (i % 32)) & 1u);
        dist += (xbit != mbit);
      }
      if (dist < dmin) dmin = dist;
    }
    return -((real)e->beta / (real)n) * (real)dmin;
  }
  {
    int N = e->lattice_n, sum = 0;
    for (int r = 0; r < N; ++r)
      for (int c = 0; c < N; ++c) {
        int x = s[r * N + c];
        sum += x * s[r * N + (c + 1) % N];
        sum += x * s[((r + 1) % N) * N + c];
      }
    return (real)e->coupling * (real)sum;
  }
}

int oracle_log_reward(const oracle_env* e, const int32_t* state, real* out) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(e, &sd, &od, &na, &ms)) return -1;
  int s[MAX_STATE];
  for (int i = 0; i < sd; ++i) s[i] = state[i];
  *out = env_log_reward(e, s, sd);
  return 0;
}

/* ------------------------------------------------------------------- MLP */

typedef struct {
  real *z1, *h1, *z2, *h2, *logit, *logp;
} act_buf;

static act_buf act_alloc(const oracle_mlp* m) {
  act_buf a;
  a.z1 = (real*)malloc(sizeof(real) * m->h1);
  a.h1 = (real*)malloc(sizeof(real) * m->h1);
  a.z2 = (real*)malloc(sizeof(real) * m->h2);
  a.h2 = (real*)malloc(sizeof(real) * m->h2);
  a.logit = (real*)malloc(sizeof(real) * m->n_actions);
  a.logp = (real*)malloc(sizeof(real) * m->n_actions);
  return a;
}
static void act_free(act_buf* a) {
  free(a->z1); free(a->h1); free(a->z2); free(a->h2); free(a->logit); free(a->logp);
}

static void mlp_forward(const oracle_mlp* m, const int* rows, int nrows, act_buf* a) {
  for (int j = 0; j < m->h1; ++j) a->z1[j] = m->b1[j];
  for (int r = 0; r < nrows; ++r) {
    const real* w = m->W1 + (size_t)rows[r] * m->h1;
    for (int j = 0; j < m->h1; ++j) a->z1[j] += w[j]; /* x_i = 1 on the active rows, 0 elsewhere */
  }
  for (int j = 0; j < m->h1; ++j) a->h1[j] = a->z1[j] > 0 ? a->z1[j] : 0;
  for (int j = 0; j < m->h2; ++j) a->z2[j] = m->b2[j];
  for (int i = 0; i < m->h1; ++i) {
    const real* w = m->W2 + (size_t)i * m->h2;
    real x = a->h1[i];
    for (int j = 0; j < m->h2; ++j) a->z2[j] += x * w[j];
  }
  for (int j = 0; j < m->h2; ++j) a->h2[j] = a->z2[j] > 0 ? a->z2[j] : 0;
  for (int j = 0; j < m->n_actions; ++j) a->logit[j] = m->b3[j];
  for (int i = 0; i < m->h2; ++i) {
    const real* w = m->W3 + (size_t)i * m->n_actions;
    real x = a->h2[i];
    for (int j = 0; j < m->n_actions; ++j) a->logit[j] += x * w[j];
  }
}

/* log-softmax restricted to the valid actions; invalid entries are set to 0 and never read */
static void masked_log_softmax(const real* logit, const int* valid, int n, real* logp) {
  int first = 1;
  real mx = 0;
  for (int a = 0; a < n; ++a)
    if (valid[a] && (first || logit[a] > mx)) { mx = logit[a]; first = 0; }
  real sum = 0;
  for (int a = 0; a < n; ++a)
    if (valid[a]) sum += rexp(logit[a] - mx);
  real lse = rlog(sum);
  for (int a = 0; a < n; ++a) logp[a] = valid[a] ? (logit[a] - mx) - lse : 0;
}

int oracle_policy_logits(const oracle_env* e, const oracle_mlp* m, const int32_t* state, real* logit, real* logp, int32_t* valid_out) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(e, &sd, &od, &na, &ms)) return -1;
  if (na != m->n_actions || od != m->in_dim) return -2;
  int s[MAX_STATE], rows[MAX_STATE], valid[MAX_ACT];
  int t = 0;
  for (int i = 0; i < sd; ++i) {
    s[i] = state[i];
    if (e->kind == ENV_BITSEQ || e->kind == ENV_BITSEQ_NA) t += (s[i] != (1 << e->k_bits));
    if (e->kind == ENV_ISING) t += (s[i] != 0);
  }
  act_buf a = act_alloc(m);
  int nr = env_obs_rows(e, s, sd, rows);
  mlp_forward(m, rows, nr, &a);
  env_valid(e, s, t, na, valid);
  masked_log_softmax(a.logit, valid, na, a.logp);
  for (int i = 0; i < na; ++i) { logit[i] = a.logit[i]; logp[i] = a.logp[i]; valid_out[i] = valid[i]; }
  act_free(&a);
  return 0;
}

/* --------------------------------------------------------------- rollout */

typedef struct {
  const oracle_env* env;
  const oracle_mlp* mlp;
  uint64_t seed, iteration;
  int32_t b_offset;         /* global index of column 0 of the buffers */
  int32_t batch, max_steps; /* buffer shapes */
  act_t* actions;         /* [max_steps][batch] */
  int32_t* length;          /* [batch] */
  int8_t* terminal_state;   /* [state_dim][batch] */
  real *log_pf, *log_pb, *log_reward;
  real epsilon;             /* probability of replacing the policy's draw by a uniform one over the valid actions */
  /* replay only */
  int replay;
  real tie_tol;
  int32_t* near_ties;  /* [batch] steps where the given action was not the argmax but within tie_tol */
  int32_t* violations; /* [batch] steps where the given action was invalid or further than tie_tol from the argmax */
  real* min_margin;    /* [batch] smallest top-2 gap of the perturbed logits seen along the trajectory */
  int b_begin, b_end;  /* column range of this worker */
} rollout_job;

static void* rollout_worker(void* arg) {
  rollout_job* J = (rollout_job*)arg;
  const oracle_env* e = J->env;
  const oracle_mlp* m = J->mlp;
  int32_t sd, od, na, ms;
  oracle_env_dims(e, &sd, &od, &na, &ms);
  act_buf A = act_alloc(m);
  int s[MAX_STATE], rows[MAX_STATE], valid[MAX_ACT];
  real pert[MAX_ACT];
  for (int col = J->b_begin; col < J->b_end; ++col) {
    uint32_t b = (uint32_t)(J->b_offset + col);
    env_reset(e, s, sd);
    real lpf = 0, lpb = 0, logr = 0, minmargin = (real)1e30;
    int len = 0, ties = 0, viol = 0;
    int steps_given = J->replay ? J->length[col] : ms;
    if (steps_given > J->max_steps) steps_given = J->max_steps;
    if (!J->replay)
      for (int t = 0; t < J->max_steps; ++t) J->actions[(size_t)t * J->batch + col] = ACT_PAD;
    for (int t = 0; t < steps_given; ++t) {
      int nr = env_obs_rows(e, s, sd, rows);
      mlp_forward(m, rows, nr, &A);
      env_valid(e, s, t, na, valid);
      masked_log_softmax(A.logit, valid, na, A.logp);
      int best = -1, second = -1;
      for (int a = 0; a < na; ++a) {
        pert[a] = A.logit[a] + action_noise(J->seed, J->iteration, b, (uint32_t)t, a);
        if (!valid[a]) continue;
        if (best < 0 || pert[a] > pert[best]) { second = best; best = a; }
        else if (second < 0 || pert[a] > pert[second]) second = a;
      }
      /* epsilon-uniform exploration (Appendix "Bit sequences", experimental setting): with probability epsilon
       * the action is uniform over the valid ones instead of drawn from P_F.  Both draws come from one more
       * Philox call per step, counter (b, t, 0xFFFFFFFE, iteration): word 0 decides (u < epsilon, compared in
       * binary32), word 1 picks the j-th valid action in increasing order, j = floor(w * n / 2^32). */
      int forced = -1;
      if (J->epsilon > 0) {
        uint32_t ctr[4] = {b, (uint32_t)t, 0xFFFFFFFEu, (uint32_t)(J->iteration & 0xFFFFFFFFu)};
        uint32_t key[2] = {(uint32_t)(J->seed & 0xFFFFFFFFu), (uint32_t)(J->seed >> 32)};
        uint32_t out[4];
        oracle_philox4x32_10(ctr, key, out);
        const float u = ((float)(out[0] >> 9) + 0.5f) * (1.0f / 8388608.0f);
        if (u < (float)J->epsilon) {
          int nvalid = 0;
          for (int a = 0; a < na; ++a) nvalid += valid[a] != 0;
          int j = (int)(((uint64_t)out[1] * (uint64_t)nvalid) >> 32);
          for (int a = 0; a < na; ++a)
            if (valid[a] && j-- == 0) { forced = a; break; }
        }
      }
      if (forced < 0 && second >= 0 && pert[best] - pert[second] < minmargin) minmargin = pert[best] - pert[second];
      int act = forced >= 0 ? forced : best;
      if (J->replay) {
        act = J->actions[(size_t)t * J->batch + col];
        if (act >= na || !valid[act]) { viol++; break; }
        if (forced >= 0) {
          if (act != forced) viol++; /* an integer decision: no tolerance */
        } else if (act != best) {
          if (pert[best] - pert[act] < J->tie_tol) ties++; else viol++;
        }
      } else {
        J->actions[(size_t)t * J->batch + col] = (act_t)act;
      }
      lpf += A.logp[act];
      int term = env_step(e, s, sd, t, act);
      lpb += env_log_pb(e, s, sd, t, act);
      len = t + 1;
      if (term) { logr = env_log_reward(e, s, sd); break; }
      if (J->replay && t + 1 == steps_given) viol++; /* given sequence ends before a terminal state */
    }
    if (J->replay) {
      J->near_ties[col] = ties;
      J->violations[col] = viol;
    } else {
      J->length[col] = len;
    }
    if (J->min_margin) J->min_margin[col] = minmargin;
    J->log_pf[col] = lpf;
    J->log_pb[col] = lpb;
    J->log_reward[col] = logr;
    for (int i = 0; i < sd; ++i) J->terminal_state[(size_t)i * J->batch + col] = (int8_t)s[i];
  }
  act_free(&A);
  return NULL;
}

static int run_rollout(rollout_job* base, int nthreads) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(base->env, &sd, &od, &na, &ms)) return -1;
  if (na != base->mlp->n_actions || od != base->mlp->in_dim) return -2;
  if (sd > MAX_STATE || na > MAX_ACT) return -3;
  if (!base->replay && base->max_steps < ms) return -4;
  if (nthreads < 1) nthreads = 1;
  if (nthreads > base->batch) nthreads = base->batch > 0 ? base->batch : 1;
  pthread_t* th = (pthread_t*)malloc(sizeof(pthread_t) * nthreads);
  rollout_job* jobs = (rollout_job*)malloc(sizeof(rollout_job) * nthreads);
  for (int k = 0; k < nthreads; ++k) {
    jobs[k] = *base;
    jobs[k].b_begin = (int)((int64_t)base->batch * k / nthreads);
    jobs[k].b_end = (int)((int64_t)base->batch * (k + 1) / nthreads);
    if (nthreads == 1) rollout_worker(&jobs[k]);
    else pthread_create(&th[k], NULL, rollout_worker, &jobs[k]);
  }
  if (nthreads > 1)
    for (int k = 0; k < nthreads; ++k) pthread_join(th[k], NULL);
  free(th);
  free(jobs);
  return 0;
}

/* Samples `batch` trajectories with global indices b_offset .. b_offset+batch-1. */
int oracle_rollout(const oracle_env* env, const oracle_mlp* mlp, uint64_t seed, uint64_t iteration, int32_t b_offset,
                   int32_t batch, int32_t max_steps, act_t* actions, int32_t* length, int8_t* terminal_state,
                   real* log_pf, real* log_pb, real* log_reward, real* min_margin, real epsilon, int nthreads) {
  rollout_job J;
  memset(&J, 0, sizeof(J));
  J.env = env; J.mlp = mlp; J.seed = seed; J.iteration = iteration; J.b_offset = b_offset;
  J.batch = batch; J.max_steps = max_steps; J.actions = actions; J.length = length;
  J.terminal_state = terminal_state; J.log_pf = log_pf; J.log_pb = log_pb; J.log_reward = log_reward;
  J.min_margin = min_margin; J.epsilon = epsilon;
  return run_rollout(&J, nthreads);
}

/* Follows the given actions (length[] steps per column) and reports, per column, the
 * trajectory scalars along THOSE actions, the number of steps where the given action is
 * not this implementation's argmax but within tie_tol of it (near ties), and the number
 * of steps where it is invalid or further away (violations).  With epsilon > 0 the steps
 * where the exploration draw decides must carry exactly the action it picks. */
int oracle_replay(const oracle_env* env, const oracle_mlp* mlp, uint64_t seed, uint64_t iteration, int32_t b_offset,
                  int32_t batch, int32_t max_steps, const act_t* actions, const int32_t* length,
                  int8_t* terminal_state, real* log_pf, real* log_pb, real* log_reward, real tie_tol,
                  int32_t* near_ties, int32_t* violations, real* min_margin, real epsilon, int nthreads) {
  rollout_job J;
  memset(&J, 0, sizeof(J));
  J.env = env; J.mlp = mlp; J.seed = seed; J.iteration = iteration; J.b_offset = b_offset;
  J.batch = batch; J.max_steps = max_steps; J.actions = (act_t*)actions; J.length = (int32_t*)length;
  J.terminal_state = terminal_state; J.log_pf = log_pf; J.log_pb = log_pb; J.log_reward = log_reward;
  J.replay = 1; J.tie_tol = tie_tol; J.near_ties = near_ties; J.violations = violations; J.min_margin = min_margin;
  J.epsilon = epsilon;
  return run_rollout(&J, nthreads);
}

/* ------------------------------------------------------- TB loss + gradient */

typedef struct {
  const oracle_env* env;
  const oracle_mlp* mlp;
  int32_t batch, max_steps;
  const act_t* actions;
  const int32_t* length;
  real log_z;
  real* delta; /* [batch] */
  oracle_grad g; /* private accumulators of this worker */
  int b_begin, b_end;
  int status;
  real kink_tol;   /* hidden units with |z| < kink_tol * (|bias| + sum |terms of z|) sit on the ReLU kink */
  real slack[6];   /* per tensor (dW1,db1,dW2,db2,dW3,db3): bound on the change if those units' masks flipped */
  int64_t n_kink;
  /* ReLU' decisions of another implementation, one byte (0 / 1) per (transition, hidden unit): transition t of
   * column col is row first[col] + t of relu1 [.][h1] and relu2 [.][h2].  NULL: this implementation's own. */
  const uint8_t *relu1, *relu2;
  const int64_t* first;
  int64_t followed, flipped, mismatched;
} grad_job;

static size_t n_w1(const oracle_mlp* m) { return (size_t)m->in_dim * m->h1; }
static size_t n_w2(const oracle_mlp* m) { return (size_t)m->h1 * m->h2; }
static size_t n_w3(const oracle_mlp* m) { return (size_t)m->h2 * m->n_actions; }

/* ReLU'(z) of one hidden unit.  Own decision: z > 0.  A decision given by another implementation is followed only
 * where the sign of z is not decidable in binary32, |z| < kink_tol * mag with mag = |bias| + sum |terms of z|
 * (the scale of the rounding error of the dot product); elsewhere the given decision must equal z > 0 and a
 * different one is counted in *mismatched and ignored.  mag is only evaluated (by the caller-supplied lazily
 * computed value) when it can matter: the given bit differs, or |z| < 1e-3. */
typedef struct { int64_t followed, flipped, mismatched; } relu_counts;

static int relu_decision(real z, int given, int have_given, real kink_tol, real mag, relu_counts* c) {
  const int own = z > 0;
  if (!have_given) return own;
  const int in_zone = rabs(z) < kink_tol * mag;
  if (in_zone) {
    c->followed++;
    if (given != own) c->flipped++;
    return given;
  }
  if (given != own) c->mismatched++;
  return own;
}

static void* grad_worker(void* arg) {
  grad_job* J = (grad_job*)arg;
  const oracle_env* e = J->env;
  const oracle_mlp* m = J->mlp;
  int32_t sd, od, na, ms;
  oracle_env_dims(e, &sd, &od, &na, &ms);
  act_buf A = act_alloc(m);
  real* g3 = (real*)malloc(sizeof(real) * na);
  real* g2 = (real*)malloc(sizeof(real) * m->h2);
  real* g1 = (real*)malloc(sizeof(real) * m->h1);
  uint8_t* d1 = (uint8_t*)malloc((size_t)m->h1);
  uint8_t* d2 = (uint8_t*)malloc((size_t)m->h2);
  relu_counts rc = {0, 0, 0};
  int s[MAX_STATE], rows[MAX_STATE], valid[MAX_ACT];
  for (int col = J->b_begin; col < J->b_end; ++col) {
    int len = J->length[col];
    /* pass 1: residual of eq. (TB_loss) for this trajectory */
    env_reset(e, s, sd);
    real lpf = 0, lpb = 0, logr = 0;
    int terminal = 0;
    for (int t = 0; t < len; ++t) {
      int act = J->actions[(size_t)t * J->batch + col];
      int nr = env_obs_rows(e, s, sd, rows);
      mlp_forward(m, rows, nr, &A);
      env_valid(e, s, t, na, valid);
      if (act >= na || !valid[act]) { J->status = -5; goto done; }
      masked_log_softmax(A.logit, valid, na, A.logp);
      lpf += A.logp[act];
      terminal = env_step(e, s, sd, t, act);
      lpb += env_log_pb(e, s, sd, t, act);
      if (terminal) { logr = env_log_reward(e, s, sd); if (t + 1 != len) { J->status = -6; goto done; } }
    }
    if (!terminal) { J->status = -6; goto done; }
    real delta = J->log_z + lpf - logr - lpb;
    J->delta[col] = delta;
    /* pass 2: d/dtheta of (1/B) delta^2 = (2 delta / B) * sum_t d log p(a_t | s_t) / dtheta */
    real coef = (real)2 * delta / (real)J->batch;
    env_reset(e, s, sd);
    for (int t = 0; t < len; ++t) {
      int act = J->actions[(size_t)t * J->batch + col];
      int nr = env_obs_rows(e, s, sd, rows);
      mlp_forward(m, rows, nr, &A);
      env_valid(e, s, t, na, valid);
      masked_log_softmax(A.logit, valid, na, A.logp);
      /* ReLU' of every hidden unit on this transition (see relu_decision) */
      for (int k = 0; k < m->h2; ++k) {
        const int have = J->relu2 != NULL;
        const int given = have ? (J->relu2[(size_t)(J->first[col] + t) * m->h2 + k] != 0) : 0;
        real mag = 0;
        if (have && (given != (A.z2[k] > 0) || rabs(A.z2[k]) < (real)1e-3)) {
          mag = rabs(m->b2[k]);
          for (int i = 0; i < m->h1; ++i) mag += rabs(A.h1[i] * m->W2[(size_t)i * m->h2 + k]);
        }
        d2[k] = (uint8_t)relu_decision(A.z2[k], given, have, J->kink_tol, mag, &rc);
      }
      for (int i = 0; i < m->h1; ++i) {
        const int have = J->relu1 != NULL;
        const int given = have ? (J->relu1[(size_t)(J->first[col] + t) * m->h1 + i] != 0) : 0;
        real mag = 0;
        if (have && (given != (A.z1[i] > 0) || rabs(A.z1[i]) < (real)1e-3)) {
          mag = rabs(m->b1[i]);
          for (int r = 0; r < nr; ++r) mag += rabs(m->W1[(size_t)rows[r] * m->h1 + i]);
        }
        d1[i] = (uint8_t)relu_decision(A.z1[i], given, have, J->kink_tol, mag, &rc);
      }
      for (int a = 0; a < na; ++a) g3[a] = valid[a] ? coef * ((real)(a == act) - rexp(A.logp[a])) : 0;
      for (int k = 0; k < m->h2; ++k) {
        real acc = 0;
        for (int a = 0; a < na; ++a) {
          J->g.dW3[(size_t)k * na + a] += A.h2[k] * g3[a];
          acc += m->W3[(size_t)k * na + a] * g3[a];
        }
        g2[k] = d2[k] ? acc : 0;
      }
      for (int a = 0; a < na; ++a) J->g.db3[a] += g3[a];
      for (int i = 0; i < m->h1; ++i) {
        real acc = 0;
        for (int k = 0; k < m->h2; ++k) {
          J->g.dW2[(size_t)i * m->h2 + k] += A.h1[i] * g2[k];
          acc += m->W2[(size_t)i * m->h2 + k] * g2[k];
        }
        g1[i] = d1[i] ? acc : 0;
      }
      for (int k = 0; k < m->h2; ++k) J->g.db2[k] += g2[k];
      if (J->kink_tol > 0 && !J->relu1) {
        /* ReLU'(z) is decided by the sign of z; an implementation in another precision may decide a unit
         * with |z| < kink_tol the other way.  Bound, per tensor, what such a flip changes (max-norm). */
        for (int k = 0; k < m->h2; ++k) {
          if (rabs(A.z2[k]) >= (real)1e-3) continue; /* cheap pre-filter */
          real mag = rabs(m->b2[k]);
          for (int i = 0; i < m->h1; ++i) mag += rabs(A.h1[i] * m->W2[(size_t)i * m->h2 + k]);
          if (rabs(A.z2[k]) >= J->kink_tol * mag) continue;
          real d = 0;
          for (int a = 0; a < na; ++a) d += m->W3[(size_t)k * na + a] * g3[a];
          d = rabs(d);
          real hmax = 0, wmax = 0;
          for (int i = 0; i < m->h1; ++i) {
            if (A.h1[i] > hmax) hmax = A.h1[i];
            real wv = A.z1[i] > 0 ? rabs(m->W2[(size_t)i * m->h2 + k]) : 0;
            if (wv > wmax) wmax = wv;
          }
          J->slack[2] += hmax * d; J->slack[3] += d;
          J->slack[0] += wmax * d; J->slack[1] += wmax * d;
          J->n_kink++;
        }
        for (int i = 0; i < m->h1; ++i) {
          if (rabs(A.z1[i]) >= (real)1e-3) continue;
          real mag = rabs(m->b1[i]);
          for (int r = 0; r < nr; ++r) mag += rabs(m->W1[(size_t)rows[r] * m->h1 + i]);
          if (rabs(A.z1[i]) >= J->kink_tol * mag) continue;
          real d = 0;
          for (int k = 0; k < m->h2; ++k) d += m->W2[(size_t)i * m->h2 + k] * g2[k];
          d = rabs(d);
          J->slack[0] += d; J->slack[1] += d;
          J->n_kink++;
        }
      }
      for (int r = 0; r < nr; ++r)
        for (int i = 0; i < m->h1; ++i) J->g.dW1[(size_t)rows[r] * m->h1 + i] += g1[i];
      for (int i = 0; i < m->h1; ++i) J->g.db1[i] += g1[i];
      env_step(e, s, sd, t, act);
    }
  }
done:
  J->followed = rc.followed; J->flipped = rc.flipped; J->mismatched = rc.mismatched;
  free(g3); free(g2); free(g1); free(d1); free(d2);
  act_free(&A);
  return NULL;
}

/* Loss = mean_b delta_b^2, dlogz = dLoss/dlogZ = (2/B) sum_b delta_b, grads = dLoss/dtheta
 * (overwritten), delta_out[b] optional.  Everything is recomputed from the action bytes.
 * With kink_tol > 0 it also reports n_kink, the number of (transition, hidden unit) pairs whose
 * pre-activation z is closer to zero than kink_tol times the sum of the magnitudes of its terms (the scale
 * of the rounding error of a dot product), and slack[6], a per-tensor bound (max-norm, order
 * dW1 db1 dW2 db2 dW3 db3) on what the gradient would change by if ReLU' were decided the other way on
 * those units -- the analogue, for the derivative of the ReLU, of the near-tie margin of the sampler. */
static int tb_loss_grad_impl(const oracle_env* env, const oracle_mlp* mlp, int32_t batch, int32_t max_steps,
                             const act_t* actions, const int32_t* length, real log_z, real* loss, real* dlogz,
                             oracle_grad* grads, real* delta_out, real kink_tol, real* slack_out,
                             int64_t* n_kink_out, const uint8_t* relu1, const uint8_t* relu2, const int64_t* first,
                             int64_t* counts_out, int nthreads) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(env, &sd, &od, &na, &ms)) return -1;
  if (na != mlp->n_actions || od != mlp->in_dim) return -2;
  if (sd > MAX_STATE || na > MAX_ACT) return -3;
  if (nthreads < 1) nthreads = 1;
  if (nthreads > batch) nthreads = batch > 0 ? batch : 1;
  size_t n1 = n_w1(mlp), n2 = n_w2(mlp), n3 = n_w3(mlp);
  size_t total = n1 + mlp->h1 + n2 + mlp->h2 + n3 + na;
  real* delta = (real*)calloc((size_t)batch, sizeof(real));
  real* priv = (real*)calloc(total * nthreads, sizeof(real));
  pthread_t* th = (pthread_t*)malloc(sizeof(pthread_t) * nthreads);
  grad_job* jobs = (grad_job*)malloc(sizeof(grad_job) * nthreads);
  for (int k = 0; k < nthreads; ++k) {
    real* p = priv + total * k;
    jobs[k].env = env; jobs[k].mlp = mlp; jobs[k].batch = batch; jobs[k].max_steps = max_steps;
    jobs[k].actions = actions; jobs[k].length = length; jobs[k].log_z = log_z; jobs[k].delta = delta;
    jobs[k].g.dW1 = p; p += n1; jobs[k].g.db1 = p; p += mlp->h1;
    jobs[k].g.dW2 = p; p += n2; jobs[k].g.db2 = p; p += mlp->h2;
    jobs[k].g.dW3 = p; p += n3; jobs[k].g.db3 = p;
    jobs[k].b_begin = (int)((int64_t)batch * k / nthreads);
    jobs[k].b_end = (int)((int64_t)batch * (k + 1) / nthreads);
    jobs[k].status = 0;
    jobs[k].kink_tol = kink_tol; jobs[k].n_kink = 0;
    jobs[k].relu1 = relu1; jobs[k].relu2 = relu2; jobs[k].first = first;
    jobs[k].followed = jobs[k].flipped = jobs[k].mismatched = 0;
    for (int q = 0; q < 6; ++q) jobs[k].slack[q] = 0;
    if (nthreads == 1) grad_worker(&jobs[k]);
    else pthread_create(&th[k], NULL, grad_worker, &jobs[k]);
  }
  if (nthreads > 1)
    for (int k = 0; k < nthreads; ++k) pthread_join(th[k], NULL);
  int status = 0;
  for (int k = 0; k < nthreads; ++k) if (jobs[k].status) status = jobs[k].status;
  real* outs[6] = {grads->dW1, grads->db1, grads->dW2, grads->db2, grads->dW3, grads->db3};
  size_t sizes[6] = {n1, (size_t)mlp->h1, n2, (size_t)mlp->h2, n3, (size_t)na};
  size_t off = 0;
  for (int q = 0; q < 6; ++q) {
    for (size_t i = 0; i < sizes[q]; ++i) {
      real acc = 0;
      for (int k = 0; k < nthreads; ++k) acc += priv[total * k + off + i];
      outs[q][i] = acc;
    }
    off += sizes[q];
  }
  real sum2 = 0, sum1 = 0;
  for (int b = 0; b < batch; ++b) { sum2 += delta[b] * delta[b]; sum1 += delta[b]; }
  *loss = sum2 / (real)batch;
  *dlogz = (real)2 * sum1 / (real)batch;
  if (delta_out) memcpy(delta_out, delta, sizeof(real) * batch);
  if (slack_out)
    for (int q = 0; q < 6; ++q) { slack_out[q] = 0; for (int k = 0; k < nthreads; ++k) slack_out[q] += jobs[k].slack[q]; }
  if (n_kink_out) { *n_kink_out = 0; for (int k = 0; k < nthreads; ++k) *n_kink_out += jobs[k].n_kink; }
  if (counts_out) {
    counts_out[0] = counts_out[1] = counts_out[2] = 0;
    for (int k = 0; k < nthreads; ++k) {
      counts_out[0] += jobs[k].followed; counts_out[1] += jobs[k].flipped; counts_out[2] += jobs[k].mismatched;
    }
  }
  free(delta); free(priv); free(th); free(jobs);
  return status;
}

int oracle_tb_loss_grad(const oracle_env* env, const oracle_mlp* mlp, int32_t batch, int32_t max_steps,
                        const act_t* actions, const int32_t* length, real log_z, real* loss, real* dlogz,
                        oracle_grad* grads, real* delta_out, real kink_tol, real* slack_out, int64_t* n_kink_out,
                        int nthreads) {
  return tb_loss_grad_impl(env, mlp, batch, max_steps, actions, length, log_z, loss, dlogz, grads, delta_out,
                           kink_tol, slack_out, n_kink_out, NULL, NULL, NULL, NULL, nthreads);
}

/* The same loss and gradient with the derivative of the ReLU taken from another implementation's decisions where,
 * and only where, binary32 cannot decide it -- the analogue for ReLU' of following given actions in oracle_replay.
 * relu1 / relu2: one byte (0 / 1) per (transition, hidden unit of layer 1 / 2), transition t of column col at row
 * first[col] + t.  A given decision is used iff |z| < kink_tol * (|bias| + sum |terms of z|); everywhere else this
 * implementation's own z > 0 is used and a given decision that differs from it is a disagreement.
 * counts_out[3] = {units whose given decision was followed (counted among units with |z| < 1e-3), of which the given
 * decision differs from z > 0, disagreements outside the margin (must be 0 for a correct implementation)}. */
int oracle_tb_loss_grad_follow(const oracle_env* env, const oracle_mlp* mlp, int32_t batch, int32_t max_steps,
                               const act_t* actions, const int32_t* length, real log_z, real* loss, real* dlogz,
                               oracle_grad* grads, real kink_tol, const uint8_t* relu1, const uint8_t* relu2,
                               const int64_t* first, int64_t* counts_out, int nthreads) {
  if (!relu1 || !relu2 || !first || !counts_out) return -7;
  return tb_loss_grad_impl(env, mlp, batch, max_steps, actions, length, log_z, loss, dlogz, grads, NULL, kink_tol,
                           NULL, NULL, relu1, relu2, first, counts_out, nthreads);
}

/* ------------------------------------------------------- SubTB / DB loss + gradient */

/* Adds to G the gradient of a scalar whose derivative w.r.t. the network outputs of this step is g3[0..n_out). */
static void backprop_outputs(const oracle_mlp* m, const act_buf* A, const int* rows, int nr, const real* g3,
                             oracle_grad* G, real* g2, real* g1) {
  const int no = m->n_actions;
  for (int k = 0; k < m->h2; ++k) {
    real acc = 0;
    for (int a = 0; a < no; ++a) {
      G->dW3[(size_t)k * no + a] += A->h2[k] * g3[a];
      acc += m->W3[(size_t)k * no + a] * g3[a];
    }
    g2[k] = A->z2[k] > 0 ? acc : 0;
  }
  for (int a = 0; a < no; ++a) G->db3[a] += g3[a];
  for (int i = 0; i < m->h1; ++i) {
    real acc = 0;
    for (int k = 0; k < m->h2; ++k) {
      G->dW2[(size_t)i * m->h2 + k] += A->h1[i] * g2[k];
      acc += m->W2[(size_t)i * m->h2 + k] * g2[k];
    }
    g1[i] = A->z1[i] > 0 ? acc : 0;
  }
  for (int k = 0; k < m->h2; ++k) G->db2[k] += g2[k];
  for (int r = 0; r < nr; ++r)
    for (int i = 0; i < m->h1; ++i) G->dW1[(size_t)rows[r] * m->h1 + i] += g1[i];
  for (int i = 0; i < m->h1; ++i) G->db1[i] += g1[i];
}

/* Subtrajectory Balance (Background, eq. SubTB_loss) along given trajectories, for a network with one output more
 * than the environment has actions: outputs 0..A-1 are the policy logits, output A is log F_theta(s).
 * With phi_t = log F(s_t) for t < n and phi_n = log R(s_n), and c_t = sum_{i<=t} (log P_F(s_i|s_i-1) -
 * log P_B(s_i-1|s_i)), the residual of the pair j < k is (phi_j - c_j) - (phi_k - c_k) = u_j - u_k, so
 *   L(tau) = sum_{j<k} w_jk (u_j - u_k)^2,  w_jk = lambda^(k-j-1) / sum_{j<k} lambda^(k-j-1)
 * (the paper's lambda^(k-j) normalised to sum to one; written this way lambda = 0 is defined and keeps exactly the
 * single-transition pairs: the Detailed Balance objective, eq. DB_loss, averaged over the transitions).
 * loss = mean over the batch; grads (overwritten) hold its gradient; P_B is fixed.
 * u_out, optional: [max_steps + 1][batch], u_t of every trajectory (0 beyond its length). */
int oracle_subtb_loss_grad(const oracle_env* env, const oracle_mlp* mlp, int32_t batch, int32_t max_steps,
                           const act_t* actions, const int32_t* length, real lambda, real* loss,
                           oracle_grad* grads, real* u_out) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(env, &sd, &od, &na, &ms)) return -1;
  if (na + 1 != mlp->n_actions || od != mlp->in_dim) return -2;
  if (sd > MAX_STATE || na + 1 > MAX_ACT || max_steps > MAX_STATE) return -3;
  const int no = na + 1;
  memset(grads->dW1, 0, sizeof(real) * n_w1(mlp)); memset(grads->db1, 0, sizeof(real) * mlp->h1);
  memset(grads->dW2, 0, sizeof(real) * n_w2(mlp)); memset(grads->db2, 0, sizeof(real) * mlp->h2);
  memset(grads->dW3, 0, sizeof(real) * n_w3(mlp)); memset(grads->db3, 0, sizeof(real) * no);
  if (u_out) memset(u_out, 0, sizeof(real) * (size_t)(max_steps + 1) * batch);
  act_buf A = act_alloc(mlp);
  real* g3 = (real*)malloc(sizeof(real) * no);
  real* g2 = (real*)malloc(sizeof(real) * mlp->h2);
  real* g1 = (real*)malloc(sizeof(real) * mlp->h1);
  real u[MAX_STATE + 2], g[MAX_STATE + 2];
  int s[MAX_STATE], rows[MAX_STATE], valid[MAX_ACT];
  real total = 0;
  int status = 0;
  for (int col = 0; col < batch && !status; ++col) {
    const int n = length[col];
    if (n < 1 || n > max_steps) { status = -4; break; }
    /* pass 1: u_t along the trajectory */
    env_reset(env, s, sd);
    real c = 0;
    int terminal = 0;
    for (int t = 0; t < n; ++t) {
      const int act = actions[(size_t)t * batch + col];
      const int nr = env_obs_rows(env, s, sd, rows);
      mlp_forward(mlp, rows, nr, &A);
      env_valid(env, s, t, na, valid);
      if (act >= na || !valid[act]) { status = -5; break; }
      masked_log_softmax(A.logit, valid, na, A.logp);
      u[t] = A.logit[na] - c;
      terminal = env_step(env, s, sd, t, act);
      c += A.logp[act] - env_log_pb(env, s, sd, t, act);
      if (terminal && t + 1 != n) { status = -6; break; }
    }
    if (status) break;
    if (!terminal) { status = -6; break; }
    u[n] = env_log_reward(env, s, sd) - c;
    /* pair sum and its derivative with respect to every u_t */
    real wsum = 0;
    for (int j = 0; j < n; ++j) { real w = 1; for (int k = j + 1; k <= n; ++k) { wsum += w; w *= lambda; } }
    real L = 0;
    for (int t = 0; t <= n; ++t) g[t] = 0;
    for (int j = 0; j < n; ++j) {
      real w = 1;
      for (int k = j + 1; k <= n; ++k) {
        const real d = u[j] - u[k];
        L += (w / wsum) * d * d;
        g[j] += (real)2 * (w / wsum) * d;
        g[k] -= (real)2 * (w / wsum) * d;
        w *= lambda;
      }
    }
    total += L;
    if (u_out) for (int t = 0; t <= n; ++t) u_out[(size_t)t * batch + col] = u[t];
    /* pass 2: u_t = phi_t - c_t; log P_F of transition t -> t+1 enters c_k for every k > t with sign -1 */
    env_reset(env, s, sd);
    for (int t = 0; t < n; ++t) {
      const int act = actions[(size_t)t * batch + col];
      const int nr = env_obs_rows(env, s, sd, rows);
      mlp_forward(mlp, rows, nr, &A);
      env_valid(env, s, t, na, valid);
      masked_log_softmax(A.logit, valid, na, A.logp);
      real kappa = 0;
      for (int k = t + 1; k <= n; ++k) kappa -= g[k];
      for (int a = 0; a < na; ++a)
        g3[a] = valid[a] ? (kappa / (real)batch) * ((real)(a == act) - rexp(A.logp[a])) : 0;
      g3[na] = g[t] / (real)batch;
      backprop_outputs(mlp, &A, rows, nr, g3, grads, g2, g1);
      env_step(env, s, sd, t, act);
    }
  }
  *loss = total / (real)batch;
  free(g3); free(g2); free(g1);
  act_free(&A);
  return status;
}

/* ------------------------------------------------------------------ backward rollout */

/* Parents of state s under the structural backward actions, in increasing index order. */
static int env_backward_choices(const oracle_env* e, const int* s, int sd, int* choice) {
  int n = 0;
  if (e->kind == ENV_GRID) {
    for (int i = 0; i < sd; ++i) if (s[i] > 0) choice[n++] = i;
  } else if (e->kind == ENV_BITSEQ) {
    int last = -1; /* left-to-right scheme: only the last written position can be emptied */
    for (int i = 0; i < sd; ++i) if (s[i] != (1 << e->k_bits)) last = i;
    if (last >= 0) choice[n++] = last;
  } else if (e->kind == ENV_BITSEQ_NA) {
    for (int i = 0; i < sd; ++i) if (s[i] != (1 << e->k_bits)) choice[n++] = i; /* any filled position */
  } else {
    for (int i = 0; i < sd; ++i) if (s[i] != 0) choice[n++] = i;
  }
  return n;
}

/* Undoes the forward move that produced s at index c; returns that forward action. */
static int env_backward_step(const oracle_env* e, int* s, int c) {
  if (e->kind == ENV_GRID) { s[c] -= 1; return c; }
  if (e->kind == ENV_BITSEQ) { int a = s[c]; s[c] = 1 << e->k_bits; return a; }
  if (e->kind == ENV_BITSEQ_NA) { int a = (c << e->k_bits) + s[c]; s[c] = 1 << e->k_bits; return a; }
  { int a = 2 * c + (s[c] > 0 ? 1 : 0); s[c] = 0; return a; }
}

/* Backward rollouts ("Library Details": start at terminal states, backward step in place of the step) under
 * the fixed uniform backward policy: for trajectory b, starting from terminal_state[:, b], parents are drawn
 * until s_0 is reached.  Outputs the trajectory in FORWARD order (actions[t][b], 0xFF padding, length[b]) and
 * log P_B(tau | x) summed in the order the moves are drawn. */
int oracle_backward_rollout(const oracle_env* env, uint64_t seed, uint64_t iteration, int32_t b_offset,
                            int32_t batch, int32_t max_steps, const int8_t* terminal_state, act_t* actions,
                            int32_t* length, real* log_pb) {
  int32_t sd, od, na, ms;
  if (oracle_env_dims(env, &sd, &od, &na, &ms)) return -1;
  if (sd > MAX_STATE || max_steps < ms) return -3;
  const uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  for (int b = 0; b < batch; ++b) {
    int s[MAX_STATE], choice[MAX_STATE], rev[MAX_STATE + 1];
    for (int i = 0; i < sd; ++i) {
      s[i] = terminal_state[(size_t)i * batch + b];
      if (env->kind == ENV_BITSEQ || env->kind == ENV_BITSEQ_NA) s[i] &= 0xFF; /* tokens are unsigned bytes */
    }
    int k = 0, draws = 0;
    real lpb = 0;
    if (env->kind == ENV_GRID) rev[k++] = env->grid_dim; /* un-stop: the terminal copy has one parent */
    for (;;) {
      const int n = env_backward_choices(env, s, sd, choice);
      if (n == 0) break; /* s_0 reached */
      if (k >= max_steps) return -4;
      uint32_t ctr[4] = {(uint32_t)(b_offset + b), (uint32_t)draws, 0xFFFFFFFFu, (uint32_t)(iteration & 0xFFFFFFFFu)};
      uint32_t out[4];
      oracle_philox4x32_10(ctr, key, out);
      const int j = (int)(((uint64_t)out[0] * (uint64_t)n) >> 32);
      lpb += -rlog((real)n);
      rev[k++] = env_backward_step(env, s, choice[j]);
      ++draws;
    }
    length[b] = k;
    for (int t = 0; t < max_steps; ++t) actions[(size_t)t * batch + b] = t < k ? (act_t)rev[k - 1 - t] : ACT_PAD;
    log_pb[b] = lpb;
  }
  return 0;
}

/* Monte-Carlo estimate of log P_theta(x) (Appendix "Bit sequences", estimator equation): for state x with
 * samples i = 0..N-1 stored at index x * N + i,  out[x] = log( (1/N) sum_i exp(log_pf - log_pb) ). */
int oracle_log_prob_estimate(const real* log_pf, const real* log_pb, int32_t n_states, int32_t n_samples, real* out) {
  if (n_states < 0 || n_samples < 1) return -1;
  for (int x = 0; x < n_states; ++x) {
    const real* f = log_pf + (size_t)x * n_samples;
    const real* bk = log_pb + (size_t)x * n_samples;
    real mx = f[0] - bk[0];
    for (int i = 1; i < n_samples; ++i) if (f[i] - bk[i] > mx) mx = f[i] - bk[i];
    real acc = 0;
    for (int i = 0; i < n_samples; ++i) acc += rexp((f[i] - bk[i]) - mx);
    out[x] = mx + rlog(acc / (real)n_samples);
  }
  return 0;
}

/* ------------------------------------------------------------------ optimiser */

static real rsqrt_(real x) { return sizeof(real) == 4 ? (real)sqrtf((float)x) : (real)sqrt((double)x); }

/* One Adam update of n parameters in place (Kingma & Ba 2015, Algorithm 1; settings: Appendix "Hypergrid",
 * hyperparameter table).  t is the 1-based count of this update; m and v are the running first and second
 * moments (zero before the first update):
 *   m <- beta1 m + (1 - beta1) g,   v <- beta2 v + (1 - beta2) g^2,
 *   theta <- theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps). */
int oracle_adam_step(real* theta, const real* g, real* m, real* v, int64_t n, int64_t t, real lr, real beta1,
                     real beta2, real eps) {
  if (!theta || !g || !m || !v || n < 0 || t < 1) return -1;
  const real c1 = (real)1 - (real)pow((double)beta1, (double)t);
  const real c2 = (real)1 - (real)pow((double)beta2, (double)t);
  for (int64_t i = 0; i < n; ++i) {
    m[i] = beta1 * m[i] + ((real)1 - beta1) * g[i];
    v[i] = beta2 * v[i] + ((real)1 - beta2) * (g[i] * g[i]);
    const real mhat = m[i] / c1;
    const real vhat = v[i] / c2;
    theta[i] = theta[i] - lr * mhat / (rsqrt_(vhat) + eps);
  }
  return 0;
}

int oracle_real_bytes(void) { return (int)sizeof(real); }

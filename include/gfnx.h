/*
 * gfnx.h -- C ABI of libgfnx_hip.so: batched on-device GFlowNet trajectory rollout and the
 * Trajectory-Balance (TB) loss with its gradient, for AMD gfx950 (MI355X).
 *
 * Vocabulary follows the paper (arXiv 2511.16592): trajectories tau = (s_0 .. s_n), forward policy
 * P_F, backward policy P_B, reward R, normalising constant Z (Background section).  An environment
 * is stateless: reset gives s_0, a step maps (state, action) to the child state and emits the
 * log-reward on the terminal transition only ("Library Details", implementation notes and usage
 * listing).  The three environments are the hypergrid (Appendix "Hypergrid"), bit sequences in the
 * autoregressive fixed-length scheme and in the non-autoregressive scheme (Appendix "Sequential environments" /
 * "Bit sequences") and the Ising partial-assignment environment (Appendix "Ising model").
 *
 * General rules for every call
 *   - returns GFNX_OK (0) or a negative gfnx_status; never throws, aborts or synchronises;
 *   - arguments are validated on the host before anything is launched (testable without a GPU);
 *   - descriptors (gfnx_env_desc, gfnx_mlp, gfnx_traj, gfnx_mlp_grad) are HOST structs, read
 *     during the call and not retained; every pointer INSIDE them is a DEVICE pointer owned by the
 *     caller; the library allocates no device memory and owns nothing between calls;
 *   - all work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default stream);
 *     buffers must stay valid until that work has completed;
 *   - all floating point is IEEE binary32.
 *
 * Conventions (the same ones the CPU reference of the test-suite follows)
 *   policy    logits = W3^T relu(W2^T relu(W1^T onehot(s) + b1) + b2) + b3, W row-major [in][out].
 *   one-hot   grid: H*i + x_i;  bitseq: (2^k+1)*pos + tok, tok = 2^k for "empty";
 *             Ising: 3*site + (x+1), x = 0 for an unassigned site, site = row*N + col.
 *   actions   grid: a < d increments coordinate a (masked when x_a = H-1), a = d stops (last
 *             index, as in the paper's usage listing);  bitseq: step t writes token a at position t;
 *             Ising: site = a/2, spin = 2*(a%2)-1, masked once the site is assigned;  bitseq_na: position = a / 2^k,
 *             word = a % 2^k, masked once the position is filled.
 *   sampling  Gumbel-max over the valid actions: argmax_a (logit_a + g_a), lowest index on ties,
 *             g = -log(-log(u)), u = ((w >> 9) + 0.5) * 2^-23, w = word (a % 4) of
 *             Philox4x32-10(counter = (b, t, a / 4, iteration lo32), key = (seed lo32, seed hi32)),
 *             b = global trajectory index, t = step.  The random draws of a trajectory do not depend
 *             on the batch it is in; its floating-point sums may be rounded in a different order
 *             (relative differences of 1e-7) when the trajectories running beside it differ.
 *   log P_B   uniform over parents: grid increment -log #{i : child_i > 0}, grid stop 0,
 *             bitseq 0, Ising and bitseq_na -log(t+1).
 */
#ifndef GFNX_H
#define GFNX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GFNX_OK = 0,
  GFNX_E_NULL = -1,        /* a required pointer is NULL */
  GFNX_E_BAD_ENV = -2,     /* environment descriptor is inconsistent */
  GFNX_E_BAD_SHAPE = -3,   /* MLP / trajectory shapes do not match the environment */
  GFNX_E_WORKSPACE = -4,   /* workspace missing, misaligned (256 B) or too small */
  GFNX_E_UNSUPPORTED = -5, /* valid request outside what the kernels are built for */
  GFNX_E_HIP = -6          /* a HIP runtime call or kernel launch failed */
} gfnx_status;

typedef enum { GFNX_ENV_GRID = 0, GFNX_ENV_BITSEQ = 1, GFNX_ENV_ISING = 2, GFNX_ENV_BITSEQ_NA = 3 } gfnx_env_kind;

/* Environment + reward descriptor (host struct, copied by value during the call).
 *   grid   : grid_dim d in 1..16, grid_side H in 2..127; reward of the Appendix "Hypergrid" equation,
 *            R = r0 + r1 * prod_i [0.25 < |x_i/(H-1) - 0.5|] + r2 * prod_i [0.3 < |.| < 0.4], strict.
 *   bitseq : n_bits = k_bits * L with k_bits in 1..8 and L <= 32; modes_dev points to DEVICE memory,
 *            n_modes x ceil(n_bits/32) uint32 words, string bit i in bit (i % 32) of word i / 32;
 *            token bits are laid out most-significant first; R = exp(-beta * min_m Hamming / n_bits)
 *            (Appendix "Bit sequences").
 *   ising  : lattice_n N in 3..10 (N*N <= 100 sites, periodic), R = exp(coupling * sum over the 2*N*N
 *            nearest-neighbour bonds of x_i x_j), each bond counted once (Appendix "Ising model",
 *            energy equation with J = (coupling/2) * adjacency).
 *   bitseq_na : the same strings, modes and reward as bitseq in the non-autoregressive scheme of Appendix
 *            "Sequential environments" (the one the paper's bit-sequence experiments use): an action picks an empty
 *            position and the k-bit word written there, a = position * 2^k + word, L * 2^k actions, masked once
 *            the position is filled; L steps; log P_B = -log(t+1) (uniform over the filled positions of the
 *            child).  Up to 256 actions (e.g. n_bits = 64, k_bits = 4) everything works as for the other kinds.
 *            Larger instances (the paper's own: n = 120, k = 8, 3840 actions) must have a multiple of 256 actions,
 *            at most 8192, and use the 16-bit action plane gfnx_traj.actions16.
 * Fields of the other kinds are ignored. */
typedef struct {
  int32_t kind;
  int32_t grid_dim, grid_side;
  float r0, r1, r2;
  int32_t n_bits, k_bits, n_modes;
  const uint32_t* modes_dev;
  float beta;
  int32_t lattice_n;
  float coupling;
} gfnx_env_desc;

/* Policy network In -> h1 -> h2 -> n_actions with ReLU (the paper's "MLP with 2 hidden layers").
 * Device pointers, row-major [in][out], biases [out].  h1 and h2 must be multiples of 64 and at most
 * 512; n_actions at most 256, except for the non-autoregressive bit sequences (see gfnx_env_desc). */
typedef struct {
  int32_t in_dim, h1, h2, n_actions;
  const float *W1, *b1, *W2, *b2, *W3, *b3;
} gfnx_mlp;

/* Networks with a flow output (hypergrid only): n_actions may be the environment's number of actions PLUS ONE.
 * The last output is then log F_theta(s), the state flow of the Detailed / Subtrajectory Balance objectives
 * (Background, eq. DB_loss, eq. SubTB_loss); sampling ignores it, gfnx_rollout / gfnx_rollout_explore / gfnx_replay
 * record it per transition in the workspace, and gfnx_subtb_loss_grad (not gfnx_tb_loss_grad) consumes it. */

/* Gradient buffers, same shapes as the weights, device pointers; OVERWRITTEN (not accumulated). */
typedef struct {
  float *dW1, *db1, *dW2, *db2, *dW3, *db3;
} gfnx_mlp_grad;

/* Structure-of-arrays trajectory batch, device pointers, caller-allocated.
 *   actions        [max_steps][batch] one byte per transition, coalesced over the batch, the buffer 4-byte
 *                  aligned; entries with
 *                  t >= length[b] are 0xFF padding (use length[], not the sentinel: 0xFF is also the
 *                  valid action 255 of an environment with 256 actions);
 *   length         [batch] number of transitions including the terminating one;
 *   terminal_state [state_dim][batch] grid coordinate / token byte / spin of the terminal state;
 *   log_pf, log_pb [batch] sums over the trajectory of log P_F(s_t | s_t-1) and log P_B(s_t-1 | s_t)
 *                  (Background, eq. forward_backward_traj);
 *   log_reward     [batch] log R of the terminal state;
 *   actions16      [max_steps][batch] the same plane in 16 bits per transition (padding 0xFFFF, 4-byte aligned), used
 *                  INSTEAD of `actions` (which may then be NULL) by environments with more than 256 actions
 *                  (gfnx_env_dims); ignored, and may be NULL, otherwise. */
typedef struct {
  int32_t batch, max_steps;
  uint8_t* actions;
  int32_t* length;
  int8_t* terminal_state;
  float *log_pf, *log_pb, *log_reward;
  uint16_t* actions16;
} gfnx_traj;

/* Host-only: sizes implied by an environment descriptor.  max_steps is the longest possible
 * trajectory: d*(H-1)+1 (grid), n_bits/k_bits (bitseq), N*N (Ising).  Any out pointer may be NULL. */
int gfnx_env_dims(const gfnx_env_desc* env, int32_t* state_dim, int32_t* obs_dim, int32_t* n_actions,
                  int32_t* max_steps);

/* Host-only: bytes of device workspace the calls below need for this environment, network and
 * batch (returns 0 if the arguments are invalid).  The workspace holds the re-laid-out weights, the
 * per-transition activations the rollout keeps for the gradient pass, and reduction partials. */
size_t gfnx_workspace_bytes(const gfnx_env_desc* env, const gfnx_mlp* mlp, int32_t batch);

/* Host-only: where, inside the workspace, a rollout (gfnx_rollout / gfnx_rollout_explore / gfnx_replay) leaves the
 * derivative of the ReLU it used on every transition -- for tools that check the gradient of eq. TB_loss against
 * another implementation, which must take the same float-decided derivative where a pre-activation is zero to
 * within binary32 rounding.  The region starts at byte *offset of the workspace and holds one row of *row_bytes
 * bytes per (step t, trajectory b) at row index t * batch + b; rows of steps t >= length[b] are undefined.  The
 * contents are valid from the end of the rollout until the next gfnx_tb_loss_grad / gfnx_subtb_loss_grad (which
 * consumes the workspace) on the same stream.
 *   GFNX_REGION_H1_SIGNS, GFNX_REGION_H2_SIGNS   one bit per hidden unit of layer 1 / 2, set iff the unit's
 *       pre-activation was > 0: unit u is bit (u % 256) / 4 of the 64-bit little-endian word 4 * (u / 256) + u % 4
 *       of the row.  GFNX_REGION_H2_SIGNS is GFNX_E_UNSUPPORTED for networks of at most 16 outputs with h2 = 256,
 *       which record no such bits: there the sign is that of the stored activation, GFNX_REGION_H2_ROWS.
 *   GFNX_REGION_H2_ROWS   h2 binary32 values per row: the post-ReLU activations of layer 2.
 * Errors: NULL pointers, descriptor / shape errors as gfnx_workspace_bytes, unknown region (GFNX_E_BAD_SHAPE). */
typedef enum { GFNX_REGION_H1_SIGNS = 0, GFNX_REGION_H2_SIGNS = 1, GFNX_REGION_H2_ROWS = 2 } gfnx_region;
int gfnx_workspace_region(const gfnx_env_desc* env, const gfnx_mlp* mlp, int32_t batch, int32_t region,
                          size_t* offset, size_t* row_bytes);

/* Forward rollout (the paper's forward_rollout utility, "Library Details"): samples `traj->batch`
 * complete trajectories from P_F given by `mlp`, starting at s_0, and fills every array of `traj`.
 * Trajectory b uses the Philox counters (b, t, ., iteration).  Also leaves in `workspace` what
 * gfnx_tb_loss_grad needs.  traj->max_steps must be >= the environment's max_steps.
 * Errors: NULL pointers, shape mismatches, unsupported sizes, workspace too small / misaligned. */
int gfnx_rollout(const gfnx_env_desc* env, const gfnx_mlp* mlp, uint64_t seed, uint64_t iteration,
                 gfnx_traj* traj, void* workspace, size_t workspace_bytes, void* hip_stream);

/* gfnx_rollout with epsilon-uniform exploration (Appendix "Bit sequences", experimental setting; the paper uses
 * epsilon = 1e-3): at every step, with probability epsilon the action is uniform over the valid actions instead of
 * drawn from P_F.  One more Philox call per step, counter (b, t, 0xFFFFFFFE, iteration lo32): word 0 -> u as above,
 * explore iff u < epsilon (binary32 comparison); word 1 picks the j-th valid action in increasing order,
 * j = floor(w * n / 2^32).  log_pf remains the log-probability under P_F of the actions taken (what the
 * Trajectory-Balance objective needs for off-policy trajectories).  epsilon = 0 is gfnx_rollout bit for bit.
 * Errors: as gfnx_rollout; epsilon outside [0, 1] or NaN is GFNX_E_BAD_SHAPE. */
int gfnx_rollout_explore(const gfnx_env_desc* env, const gfnx_mlp* mlp, uint64_t seed, uint64_t iteration,
                         float epsilon, gfnx_traj* traj, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Teacher-forced rollout: follows the given traj->actions / traj->length (inputs) instead of
 * sampling, and fills log_pf, log_pb, log_reward, terminal_state and the workspace exactly as
 * gfnx_rollout would (off-policy trajectories, the trajectory distributions of eq.
 * forward_backward_traj for given tau).  A given action that is impossible in its state cuts that
 * trajectory there (no transition, log_reward 0), and a sequence that does not reach a terminal state within
 * length[b] steps ends with log_reward 0: both are memory-safe, but the loss and gradient contributions of
 * such a trajectory are unspecified. */
int gfnx_replay(const gfnx_env_desc* env, const gfnx_mlp* mlp, gfnx_traj* traj, void* workspace,
                size_t workspace_bytes, void* hip_stream);

/* Trajectory-Balance loss (Background, eq. TB_loss) averaged over the batch and its gradient:
 *   delta_b = log_z + log_pf[b] - log_reward[b] - log_pb[b],   loss = mean_b delta_b^2,
 *   *dlogz_dev = d loss / d log Z = (2/B) sum_b delta_b,   grads = d loss / d (W1 .. b3), with P_B fixed.
 * `traj`, `mlp`, `env`, `workspace` must be the ones of the immediately preceding gfnx_rollout or
 * gfnx_replay on the same stream: the per-transition activations are taken from the workspace and are
 * consumed (overwritten) by this call, so it can run once per rollout.  loss_dev and dlogz_dev are
 * device pointers to one float each. */
int gfnx_tb_loss_grad(const gfnx_env_desc* env, const gfnx_mlp* mlp, const gfnx_traj* traj, float log_z,
                      float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* Subtrajectory Balance loss (Background, eq. SubTB_loss) and its gradient, for a network with a flow output
 * (see gfnx_mlp) on the hypergrid, along the trajectories of the immediately preceding gfnx_rollout /
 * gfnx_rollout_explore / gfnx_replay on the same stream and workspace (consumed, as by gfnx_tb_loss_grad):
 *   phi_t = log F(s_t) for t < n, phi_n = log R(s_n);  S_jk = sum_{t=j+1..k} (log P_F(s_t|s_t-1) - log P_B(s_t-1|s_t));
 *   L(tau) = sum_{0<=j<k<=n} w_jk (phi_j - phi_k + S_jk)^2,  w_jk = lambda^(k-j-1) / sum_{j<k} lambda^(k-j-1)
 * (the paper's lambda^(k-j) normalised to sum to one; in this form lambda = 0 is defined and keeps the single
 * transitions only: the Detailed Balance objective, eq. DB_loss, averaged over the transitions of a trajectory);
 * *loss_dev = mean over the batch, grads = its gradient (W3 / b3 gradients include the flow column), P_B fixed.
 * lambda in [0, 1].  Errors: as gfnx_tb_loss_grad; a network without a flow output, or another environment than
 * the hypergrid, is GFNX_E_BAD_SHAPE. */
int gfnx_subtb_loss_grad(const gfnx_env_desc* env, const gfnx_mlp* mlp, const gfnx_traj* traj, float lambda,
                         float* loss_dev, gfnx_mlp_grad* grads, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* Backward rollout ("Library Details": a rollout started at terminal states with the backward step in place of
 * the step) under the fixed uniform backward policy.  INPUT: traj->terminal_state [state_dim][batch] (grid
 * coordinates, clamped into 0..H-1; token bytes; spins, anything not positive counting as -1).  OUTPUT, for a
 * trajectory tau_b ~ P_B(. | x_b) drawn parent by parent until s_0: traj->actions (traj->actions16 beyond 256
 * actions) in FORWARD order with 0xFF (0xFFFF) padding, traj->length, traj->log_pb = log P_B(tau_b | x_b).  traj->log_pf and traj->log_reward are not touched
 * (they may be NULL); gfnx_replay on the same `traj` then evaluates log P_F along these trajectories.  Parents are
 * taken in increasing index order (grid: coordinates > 0; Ising: assigned sites; non-autoregressive bit sequences:
 * filled positions), the j-th with
 * j = floor(w * n / 2^32), w = word 0 of Philox4x32-10(counter = (b, k, 0xFFFFFFFF, iteration lo32), key = seed),
 * k = index of the backward move; moves with a single parent (the grid's un-stop, every move of the left-to-right
 * bit sequences) draw nothing.  No workspace and no network are needed; env->modes_dev is not read.
 * Errors: NULL pointers, bad descriptor, traj->max_steps below the environment's, unsupported sizes. */
int gfnx_backward_rollout(const gfnx_env_desc* env, uint64_t seed, uint64_t iteration, gfnx_traj* traj,
                          void* hip_stream);

/* Monte-Carlo estimate of the probability of sampling a terminal state (Appendix "Bit sequences", estimator
 * equation): with the n_samples trajectories of state x stored at indices x * n_samples + i,
 *   log_p_dev[x] = log( (1 / n_samples) sum_i exp(log_pf_dev[.] - log_pb_dev[.]) ),  x = 0 .. n_states-1.
 * Device pointers; log_pf from gfnx_replay, log_pb from gfnx_backward_rollout (or gfnx_replay: same value).
 * Errors: NULL pointers, n_states < 1, n_samples < 1, n_states * n_samples beyond 2^31-1. */
int gfnx_log_prob_estimate(const float* log_pf_dev, const float* log_pb_dev, int32_t n_states, int32_t n_samples,
                           float* log_p_dev, void* hip_stream);

/* Optimiser settings of a training iteration: Adam (Kingma & Ba 2015, Algorithm 1) as the paper trains with
 * (Appendix "Hypergrid", hyperparameter table: lr 1e-3, lr_log_z 1e-1, beta1 0.9, beta2 0.999, eps 1e-8, no
 * weight decay).  Host struct. */
typedef struct {
  float lr;       /* learning rate of the six weight tensors */
  float lr_log_z; /* learning rate of log Z */
  float beta1, beta2, eps;
} gfnx_adam_cfg;

/* Optimiser state: running first (m) and second (v) moments, shaped like the weights, and those of log Z.
 * Device pointers, caller-allocated, all zero before the first update. */
typedef struct {
  gfnx_mlp_grad m, v;
  float* log_z_mv; /* two floats: m and v of log Z */
} gfnx_adam_state;

/* One Adam update, in place, of the six weight tensors `mlp` points at (the const of gfnx_mlp's pointer types is
 * dropped for this call) and of *log_z_dev, from `grads` and *dlogz_dev:
 *   m <- beta1 m + (1-beta1) g,  v <- beta2 v + (1-beta2) g^2,
 *   theta <- theta - lr (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps),
 * `step` = 1-based count of this update (>= 1).  log_z_dev, dlogz_dev and state->log_z_mv may all be NULL to
 * leave log Z out.  One elementwise launch; nothing but the named buffers is read or written.
 * Errors: NULL pointers, non-positive sizes, step < 1, beta outside [0, 1), lr or eps negative. */
int gfnx_adam_step(const gfnx_mlp* mlp, float* log_z_dev, const gfnx_mlp_grad* grads, const float* dlogz_dev,
                   const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* hip_stream);

/* One whole on-policy training iteration (the loop the paper's speed table counts: rollout, objective, backward
 * pass, optimiser step), enqueued without any host round trip: gfnx_rollout with (seed, iteration), then
 * gfnx_tb_loss_grad with log Z read from *log_z_dev, then gfnx_adam_step with `step`.  Outputs as for those
 * calls: traj, *loss_dev and *dlogz_dev (of the weights BEFORE the update), grads; weights, *log_z_dev and the
 * optimiser state are updated in place.  Errors: the union of the three calls'. */
int gfnx_train_step(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                    uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                    const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/* Variants of a training iteration. */
typedef struct {
  float epsilon;      /* epsilon-uniform exploration in the rollout (gfnx_rollout_explore); 0 = on-policy */
  float subtb_lambda; /* negative: Trajectory Balance; in [0, 1]: gfnx_subtb_loss_grad with this lambda (0 = Detailed
                         Balance), for a network with a flow output on the hypergrid */
} gfnx_train_opts;

/* gfnx_train_step with the rollout and the objective chosen by `opts` (the settings the paper trains with besides
 * on-policy TB: epsilon-uniform exploration; DB and SubTB on the hypergrid).  With a Subtrajectory Balance objective
 * there is no log Z: log_z_dev, dlogz_dev and state->log_z_mv are ignored and may be NULL.
 * gfnx_train_step is this call with opts = {0, -1}.  Errors: the union of the calls it is made of; an objective
 * that does not fit the network (flow output or not) is GFNX_E_BAD_SHAPE. */
int gfnx_train_step_opts(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                         uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                         const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, const gfnx_train_opts* opts,
                         int64_t step, void* workspace, size_t workspace_bytes, void* hip_stream);

/* gfnx_train_step for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same training iteration with the workspace taken from a fixed array of
 * GFNX_STATIC_SCRATCH_BYTES that is part of the library's device code (each GPU the library runs on holds its own copy
 * until the process ends) instead of a caller-provided buffer.  The call itself allocates and frees nothing (keep
 * gfnx_timing_enable off: the timing aid creates events).  Inputs, outputs, optimiser state and results are exactly
 * those of gfnx_train_step; the calling thread's current device must be the one that holds the buffers.
 * Limits: gfnx_workspace_bytes(env, mlp, traj->batch) must not exceed GFNX_STATIC_SCRATCH_BYTES, else
 * GFNX_E_WORKSPACE is returned before anything is launched (64 MiB hold batches of 16 to 64 trajectories of every
 * configuration of the paper's three environments).  Every call on a GPU uses that GPU's one array, whose contents
 * are whatever the previous call left (nothing in it has to start at zero: each call writes what it reads): calls
 * that overlap on one GPU, on any streams, race; calls in stream order do not.
 * Errors: as gfnx_train_step; GFNX_E_WORKSPACE as above; GFNX_E_HIP if the array's address cannot be obtained. */
#define GFNX_STATIC_SCRATCH_BYTES (64u << 20)
int gfnx_train_step_static(const gfnx_env_desc* env, const gfnx_mlp* mlp, float* log_z_dev, uint64_t seed,
                           uint64_t iteration, gfnx_traj* traj, float* loss_dev, float* dlogz_dev, gfnx_mlp_grad* grads,
                           const gfnx_adam_state* state, const gfnx_adam_cfg* cfg, int64_t step, void* hip_stream);

/* Measurement aid (not part of the method; not thread-safe).  While enabled, every kernel (or small group
 * of kernels) the library launches is bracketed by HIP events recorded on the launch stream, labelled
 * "rollout", "gemm_tn_w2", ...  gfnx_timing_enable(on) also discards the records taken so far;
 * gfnx_timing_only(label) restricts recording to one label (two events per step instead of dozens).
 * gfnx_timing_labels() returns the number of labels seen; gfnx_timing_get(label, ...) WAITS for the recorded
 * events of that label (the one call of the library that synchronises) and returns how many launches were
 * recorded and their summed duration in milliseconds; *name points to static storage. */
int gfnx_timing_enable(int on);
int gfnx_timing_only(const char* label); /* record this label only (NULL or "" = every label) */
int gfnx_timing_labels(void);
int gfnx_timing_get(int label, const char** name, int32_t* launches, float* total_ms);

/* Human-readable name of a status code (static storage). */
const char* gfnx_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* GFNX_H */

/*
 * CPU oracle for the policy worker's batched actor-critic step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a slow, direct-loop,
 * fp64 restatement of what the step computes, used only by the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg.  It shares no code with the
 * HIP library and neither includes the other's headers.
 *
 * What the step is (paper, Sec. 3.1 "policy worker"): a batch of observations
 * x_t and recurrent states h_t goes in; the network pi produces the action
 * distributions mu(a_t | x_t, h_t) and the new states h_{t+1}; actions a_t are
 * sampled from mu and returned with h_{t+1}.  The network (paper, App. "Model
 * architectures"): conv encoder -> fully connected layer -> RNN core (GRU in
 * the large-scale experiments) -> one FC head for the action distribution(s)
 * and one for the baseline (value).  The full model has L independent
 * categorical heads (paper, Fig. A.1 caption and the action-space table), so
 * the joint log-probability is the sum over heads.
 *
 * The paper fixes none of the layer sizes, the normalisation, the GRU
 * convention, the reset rule or the sampler; the readings taken here are listed
 * next to each function.
 *
 * Arithmetic: inputs (weights, h_in) are fp32 and are widened to fp64; every
 * intermediate activation is fp64 with plain left-to-right summation; h_out,
 * value and logits are rounded to fp32 once, on output.  The sampler is defined
 * in fp32 on the fp32 logits (see ref_head_sample), because there a floating
 * point comparison decides an integer.
 *
 * Pins (tests/test_oracle_*.py): convolution, pooling, linear and GRU against
 * PyTorch's CPU fp64 routines and hand-computed / closed-form cases; the whole
 * step against a PyTorch fp64 composition, the pass over trajectories against
 * PyTorch's fp64 sequence modules; softmax and sampler against their
 * invariants and a chi-square test; Philox against its published known answers
 * and an independent big-integer implementation.  PARITY UNPINNED: the ResNet
 * pooling alignment, the normalisation constant and the initialisation variance
 * are conventions of this build, not of the paper.
 */
#ifndef SF_ORACLE_H
#define SF_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define REF_MAX_CONV 4
#define REF_MAX_STAGE 4
#define REF_MAX_HEADS 16
#define REF_MAX_MEAS_LAYERS 2
#define REF_MAX_CONV_TENSORS 20

/* Network description.  encoder 0: n_conv plain convolutions (each + ReLU).
 * encoder 1: n_stage residual stages (see ref_resnet_encoder). */
typedef struct {
  int32_t obs_c, obs_h, obs_w;
  int32_t encoder;
  int32_t n_conv;
  int32_t conv_cout[REF_MAX_CONV], conv_k[REF_MAX_CONV], conv_stride[REF_MAX_CONV],
      conv_pad[REF_MAX_CONV];
  int32_t n_stage;
  int32_t stage_ch[REF_MAX_STAGE];
  int32_t blocks_per_stage;
  int32_t fc_dim, rnn_dim;
  int32_t n_heads;
  int32_t head_sizes[REF_MAX_HEADS];
  float obs_sub, obs_mul; /* x = ((double)u8 - obs_sub) * obs_mul */
  int32_t rnn_type;       /* 0 GRU, 1 LSTM (state row = [h | c], 2 * rnn_dim floats) */
  int32_t meas_dim;       /* length of the measurement vector of the "full" architecture; 0 = none */
  int32_t n_meas_layers;  /* 1..REF_MAX_MEAS_LAYERS fully connected + ReLU layers on it */
  int32_t meas_hidden[REF_MAX_MEAS_LAYERS];
} ref_net;

/* fp32 parameters in their canonical layouts (all host memory, read only).
 * conv_w[i]: [cout][cin][k][k]; conv_b[i]: [cout].  Residual encoder order:
 * per stage the stage convolution, then for each block its two convolutions.
 * fc_w: [fc_dim][flat] with flat = c*(H*W) + y*W + x.  GRU: w_ih [3H][fc_dim],
 * w_hh [3H][H], b_ih [3H], b_hh [3H], gate rows ordered r, z, n.  LSTM: the same
 * four tensors with 4H rows, gate rows ordered i, f, g, o.  With a measurement
 * encoder the recurrent core's input is [fc output | encoded measurements], so
 * w_ih has fc_dim + meas_hidden[last] columns.
 * pi_w: [sum(head_sizes)][H] (heads concatenated), pi_b likewise.
 * v_w: [H], v_b: [1]. */
typedef struct {
  const float* conv_w[REF_MAX_CONV_TENSORS];
  const float* conv_b[REF_MAX_CONV_TENSORS];
  const float* fc_w;
  const float* fc_b;
  const float* rnn_w_ih;
  const float* rnn_w_hh;
  const float* rnn_b_ih;
  const float* rnn_b_hh;
  const float* pi_w;
  const float* pi_b;
  const float* v_w;
  const float* v_b;
  const float* meas_w[REF_MAX_MEAS_LAYERS]; /* [meas_hidden[l]][previous width] */
  const float* meas_b[REF_MAX_MEAS_LAYERS];
} ref_params;

/* ---- building blocks (exported so that each can be pinned on its own) ---- */

/* out[o][i][j] = bias[o] + sum_{c,p,q} w[o][c][p][q] * in[c][i*s+p-pad][j*s+q-pad],
 * reads outside the image contribute 0; Ho = floor((H + 2 pad - k)/s) + 1.
 * relu != 0 applies max(0, .) to the result.  Returns 0, or -1 if Ho or Wo < 1. */
int ref_conv2d(const double* in, int C, int H, int W, const float* w, const float* bias, int O,
               int k, int s, int pad, int relu, double* out);

/* 3x3 window, stride 2, one ring of padding that never wins the maximum:
 * output (i, j) covers input rows 2i-1..2i+1 and columns 2j-1..2j+1 clipped to
 * the image; Ho = floor((H - 1)/2) + 1. */
void ref_maxpool3x3s2p1(const double* in, int C, int H, int W, double* out);

/* out[o] = bias[o] + sum_i w[o][i] * in[i]; relu as above. */
void ref_linear(const double* in, int n_in, const float* w, const float* bias, int n_out,
                int relu, double* out);

/* GRU cell, the convention of the framework the paper was built on:
 *   r = sigma(W_ir x + b_ir + W_hr h + b_hr)
 *   z = sigma(W_iz x + b_iz + W_hz h + b_hz)
 *   n = tanh (W_in x + b_in + r * (W_hn h + b_hn))
 *   h' = (1 - z) * n + z * h
 * h is the state AFTER the episode-boundary reset (the caller zeroes it). */
void ref_gru_cell(const double* x, int n_in, const double* h, int H, const float* w_ih,
                  const float* w_hh, const float* b_ih, const float* b_hh, double* h_new);

/* LSTM cell (paper, App. "Model architectures": the benchmark model's core), the
 * convention of the framework the paper was built on:
 *   i = sigma(W_ii x + b_ii + W_hi h + b_hi)      f = sigma(W_if x + b_if + W_hf h + b_hf)
 *   g = tanh (W_ig x + b_ig + W_hg h + b_hg)      o = sigma(W_io x + b_io + W_ho h + b_ho)
 *   c' = f * c + i * g                             h' = o * tanh(c')
 * h, c are the state AFTER the episode-boundary reset. */
void ref_lstm_cell(const double* x, int n_in, const double* h, const double* c, int H,
                   const float* w_ih, const float* w_hh, const float* b_ih, const float* b_hh,
                   double* h_new, double* c_new);

/* Residual encoder (the reading of "ResNet backbone as in IMPALA"): per stage
 * conv3x3/s1/pad1 (bias, no ReLU) -> ref_maxpool3x3s2p1 -> blocks of
 * y = x + conv_b(relu(conv_a(relu(x)))) with 3x3/s1/pad1 convolutions; after the
 * last stage a ReLU.  out must hold stage_ch[last] * Hf * Wf doubles; the final
 * spatial size is returned through hf, wf. */
int ref_resnet_encoder(const ref_net* net, const ref_params* p, const double* x, double* out,
                       int* hf, int* wf);

/* Philox4x32 with 10 rounds (Salmon et al., SC'11): counter c[4], key k[2]. */
void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* u = ((w >> 9) + 0.5) * 2^-23, exact in fp32 and strictly inside (0, 1). */
float ref_bits_to_uniform(uint32_t w);
void ref_bits_to_uniform_many(const uint32_t* w, int64_t n, float* u);

/* g = -logf(-logf(u)), evaluated in fp32. */
float ref_gumbel(float u);

/* The four uniform words for categories 4*block .. 4*block+3 of one head:
 * key = (seed lo, seed hi), counter = (env, step lo, step hi, head<<16 | block). */
void ref_sampler_words(uint64_t seed, uint32_t env, uint64_t step, uint32_t head, uint32_t block,
                       uint32_t out[4]);

/* One categorical head.  logits[A] fp32.  Gumbel-max: perturbed_i = logits_i +
 * g_i in fp32, action = lowest index attaining the maximum.  logp = logits[a] -
 * (m + log sum exp(logits_i - m)) in fp64.  margin = best minus second-best
 * perturbed value (+inf when A == 1).  If g_override != NULL it replaces the
 * generated Gumbel noise (used to test the tie rule). */
void ref_head_sample(const float* logits, int A, uint64_t seed, uint32_t env, uint64_t step,
                     uint32_t head, const float* g_override, int32_t* action, double* logp,
                     float* margin);

/* Histogram of n draws of one head with fixed logits: env = 0..n_env-1 fastest,
 * step = step0 + draw / n_env. */
void ref_head_histogram(const float* logits, int A, uint64_t seed, uint32_t head, int64_t n,
                        uint32_t n_env, uint64_t step0, int64_t* counts);

/* log softmax of one head in fp64 (out[A]). */
void ref_log_softmax(const float* logits, int A, double* out);

/* ---- the whole step ------------------------------------------------------ */

/* Size of the flattened encoder output for this net, or -1 if a layer would
 * produce an empty image. */
int64_t ref_flat_size(const ref_net* net);

/* One policy step on B rows (all host pointers).
 *   obs   [B][C][H][W] u8;  meas [B][meas_dim] fp32 (NULL when meas_dim is 0: the
 *   "full" architecture's low-dimensional game information, paper, App. "VizDoom
 *   experiments");  h_in [B][state_dim];  done [B] (non-zero = this
 *   observation starts a new episode: the incoming state is zeroed BEFORE the
 *   cell, so stale state cannot reach this step's outputs)
 *   actions [B][n_heads]; logp [B] joint log-probability; value [B];
 *   h_out [B][state_dim]; logits_opt [B][sumA] or NULL; margin_opt [B][n_heads]
 *   or NULL (top-2 perturbed margin per head).
 * Sampler counter word "env" is the batch row index.  Rows are independent and
 * are spread over OpenMP threads.  Returns 0, -1 on a bad description. */
int ref_policy_step(const ref_net* net, const ref_params* p, int32_t B, const uint8_t* obs,
                    const float* meas, const float* h_in, const uint8_t* done, uint64_t seed,
                    uint64_t step, int32_t* actions, float* logp, float* value, float* h_out,
                    float* logits_opt, float* margin_opt);

/* Floats per state row: rnn_dim for a GRU, 2 * rnn_dim ([h | c]) for an LSTM. */
int ref_state_dim(const ref_net* net);

/* The same step when the batch rows are a subset of a larger population of
 * environments (paper, Sec. 3.3: components exchange indices into preallocated
 * tensors; Sec. 3.2: with double-buffered sampling the policy worker serves the
 * two halves of a worker's environments in alternation).  Row b belongs to
 * environment e = env_ids[b]:
 *   its incoming state is h_table[e] (zeroed by done[b] as above), its new
 *   state is written back to h_table[e]; rows of the table that no batch row
 *   names are left untouched; the sampler's counter word "env" is e, so what
 *   an environment draws does not depend on where in which batch it sits.
 * h_table [n_env][state_dim]; env_ids [B], distinct, each in [0, n_env).
 * Returns 0, -1 on a bad description, -2 on an id out of range or named twice
 * (nothing is written then). */
int ref_policy_step_indexed(const ref_net* net, const ref_params* p, int32_t B, const uint8_t* obs,
                            const float* meas, float* h_table, int32_t n_env, const int32_t* env_ids,
                            const uint8_t* done, uint64_t seed, uint64_t step, int32_t* actions,
                            float* logp, float* value, float* logits_opt, float* margin_opt);

/* The learner's forward pass over trajectories (paper, Sec. 3.1: the learner recomputes the
 * network's outputs on the collected trajectories of T steps, the recurrent core unrolled
 * over them; hyperparameter table of App. "VizDoom experiments": rollout T = 32).  Time-major
 * arrays: obs [T][N][C][H][W]; meas [T][N][meas_dim] or NULL; h0 [N][state_dim], the state
 * each trajectory started from; done [T][N] (non-zero at (t, n): step t of trajectory n is
 * the first of a new episode, its incoming state is zero).  It is T applications of the
 * step in order, trajectory n at time t taking the state that time t - 1 left (h0 at t = 0):
 *   logits [T][N][sumA]; value [T][N]; h_seq [T][N][state_dim] (row t = state after step t).
 * No action is drawn.  Returns 0, -1 on a bad description or T < 1. */
int ref_policy_unroll(const ref_net* net, const ref_params* p, int32_t T, int32_t N,
                      const uint8_t* obs, const float* meas, const float* h0, const uint8_t* done,
                      float* logits, float* value, float* h_seq);

/* ---- learner-side loss on a batch of trajectories -------------------------- */

/* The loss of the paper's learner (Sec. 3.4 and the hyperparameter table of App.
 * "VizDoom experiments": V-trace targets with rho_bar = c_bar = 1 combined with the PPO
 * clipping range [1/1.1, 1.1], entropy coefficient 0.003, critic-loss coefficient 0.5) on N
 * trajectories of T steps, time-major.  The paper names the two methods and cites them
 * without formulas; the formulas below are the published ones, the combination is this
 * build's reading.
 *   pi      = softmax per head of logits[t][n];  logp_pi = sum over heads of log pi(a)
 *   ratio   = exp(logp_pi - logp_mu)                       (mu: the behaviour policy)
 *   rho     = min(rho_bar, ratio),  c = min(c_bar, ratio),  g_t = gamma * (1 - done_t)
 *   delta_t = rho_t * (r_t + g_t * V_{t+1} - V_t)
 *   vs_t    = V_t + sum_{k=t}^{T-1} (prod_{i=t}^{k-1} g_i c_i) * delta_k      (V-trace target)
 *   adv_t   = r_t + g_t * vs_{t+1} - V_t        with vs_T = V_T (the bootstrap value)
 *   L_pi    = -mean( min(ratio * adv, clamp(ratio, 1/clip, clip) * adv) )
 *   L_v     = critic_coef * mean( (V_t - vs_t)^2 )
 *   L_ent   = -entropy_coef * mean( sum over heads of entropy(pi) )
 *   total   = L_pi + L_v + L_ent          (means over the T*N samples)
 * Gradients treat vs and adv as constants:
 *   dlogits = d total / d logits,  dvalues[t][n] = d L_v / d V_t  (t < T).
 * logits [T][N][sumA]; actions [T][N][n_heads]; logp_mu, rewards, dones [T][N];
 * values [T+1][N] (row T: bootstrap).  Outputs in fp64: vs, adv [T][N]; loss[4] =
 * {L_pi, L_v, L_ent, total}; dlogits [T][N][sumA] and dvalues [T][N] may be NULL.
 * Returns 0, -1 on bad sizes or an action outside its head. */
typedef struct {
  int32_t T, N, n_heads;
  int32_t head_sizes[REF_MAX_HEADS];
  float gamma, rho_bar, c_bar, clip, critic_coef, entropy_coef;
} ref_loss_cfg;

int ref_appo_loss(const ref_loss_cfg* cfg, const float* logits, const int32_t* actions,
                  const float* logp_mu, const float* values, const float* rewards,
                  const uint8_t* dones, double* vs, double* adv, double* loss, double* dlogits,
                  double* dvalues);

/* Threads ref_policy_step will use. */
int ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif

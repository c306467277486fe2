/*
 * sf_policy -- the policy worker's batched actor-critic step on one MI355X (gfx950).
 *
 * The operation (paper, Sec. 3.1, "policy worker"): a batch of observations x_t
 * and recurrent states h_t is run through the policy network, giving the action
 * distributions mu(a_t | x_t, h_t) and the new states h_{t+1}; actions a_t are
 * sampled from mu and returned together with h_{t+1}.  The network (paper, App.
 * "Model architectures"): convolutional encoder -> fully connected layer -> RNN
 * core (GRU, as in the paper's large-scale experiments) -> one linear head for
 * the action distribution(s) and one for the baseline (value).  The full action
 * space is a tuple of L independent categorical heads (paper, App. "VizDoom
 * experiments", action-space table), so the joint log-probability is the sum of
 * the per-head log-probabilities.
 *
 * The policy worker of the paper is stateless (Sec. 3.1 "Parallelism"): all
 * per-environment state lives in tensors owned by someone else.  Accordingly
 * sf_policy_step is a pure function of (weights, obs, h_in, done, seed, step):
 * row b of every output depends on row b of the inputs and on b itself (the
 * sampler's counter word) only, and is bitwise reproducible from call to call.
 *
 * Conventions
 *   - every function returns an int status (SF_OK or a negative SF_ERR_*),
 *     never throws and never aborts; sf_last_error() gives the text of the last
 *     failure on the calling thread.
 *   - "dev" pointers are device memory on the HIP device given at create time;
 *     "host" pointers are ordinary host memory.
 *   - the library copies and repacks the weights during sf_policy_create (the
 *     caller may free them as soon as it returns) and allocates its workspace
 *     there, sized for max_batch; sf_policy_step allocates nothing, does not
 *     synchronise, and keeps no pointer past the completion of the stream work
 *     it enqueues.  The caller owns every buffer passed to sf_policy_step.
 *   - one sf_policy handle must not be stepped from two threads or on two
 *     streams at the same time (its workspace is shared by its calls,
 *     sf_policy_step_indexed and sf_policy_unroll included).
 */
#ifndef SF_POLICY_H
#define SF_POLICY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SF_ABI_VERSION 2u
#define SF_MAX_CONV 4
#define SF_MAX_STAGE 4
#define SF_MAX_HEADS 16
#define SF_MAX_CONV_TENSORS 20
#define SF_MAX_MEAS_LAYERS 2

enum {
  SF_OK = 0,
  SF_ERR_ARG = -1,    /* null or misaligned pointer, bad struct_size / abi_version */
  SF_ERR_SHAPE = -2,  /* inconsistent network description (empty layer output, ...) */
  SF_ERR_BATCH = -3,  /* B < 0 or B > max_batch */
  SF_ERR_ALIAS = -4,  /* h_out overlaps h_in */
  SF_ERR_DEVICE = -5, /* a HIP call failed */
  SF_ERR_OOM = -6,    /* device allocation failed at create */
  SF_ERR_ARCH = -7    /* the device is not gfx950 */
};

enum { SF_ENCODER_CONV = 0, SF_ENCODER_RESNET = 1 };
enum { SF_DTYPE_FP32 = 0, SF_DTYPE_BF16 = 1 };
enum { SF_RNN_GRU = 0, SF_RNN_LSTM = 1 };

typedef struct sf_policy sf_policy; /* opaque */

typedef struct {
  int32_t cout, k, stride, pad; /* square kernel; out = floor((in + 2 pad - k) / stride) + 1 */
} sf_conv;

typedef struct {
  uint32_t struct_size; /* sizeof(sf_policy_config) */
  uint32_t abi_version; /* SF_ABI_VERSION */
  int32_t max_batch;    /* largest B that sf_policy_step will be given */
  int32_t obs_c, obs_h, obs_w;
  int32_t encoder; /* SF_ENCODER_CONV: n_conv convolutions, each followed by ReLU.
                      SF_ENCODER_RESNET: n_stage stages of conv3x3/s1/pad1 ->
                      maxpool 3x3/s2/pad1 (padding never wins the maximum) ->
                      blocks_per_stage residual blocks x + conv(relu(conv(relu(x))));
                      ReLU after the last stage. */
  int32_t n_conv;
  sf_conv conv[SF_MAX_CONV];
  int32_t n_stage;
  int32_t stage_ch[SF_MAX_STAGE];
  int32_t blocks_per_stage;
  int32_t fc_dim;  /* fully connected layer after the encoder, followed by ReLU */
  int32_t rnn_dim; /* hidden size H of the recurrent core */
  int32_t n_heads; /* independent categorical heads */
  int32_t head_sizes[SF_MAX_HEADS];
  int32_t dtype; /* SF_DTYPE_FP32, or SF_DTYPE_BF16: every parameter is replaced by the nearest
                    bf16 value (ties to even) of what the caller passes; encoder and FC
                    activations are 16-bit with fp32 accumulation; the recurrent state, the
                    gate arithmetic, the heads and the sampler stay fp32.  The 16-bit
                    activation type is bf16 in the plain convolution stack and fp16 in the
                    residual encoder (15 convolutions deep: 8-bit significands do not hold the
                    2e-2 tolerance there).  Limits of the fp16 case: an encoder or FC weight
                    beyond +-65280 is rejected at create (SF_ERR_ARG); a weight below 2^-14
                    in magnitude is held on fp16's subnormal grid (multiples of 2^-24); and
                    if any activation of a row's encoder exceeds 65504 in magnitude, that
                    row's outputs are unspecified (possibly finite), the other rows of the
                    batch being unaffected.  With pixel values normalised to [0, 1] and
                    weights of variance 1/fan_in the activations are of order 1. */
  float obs_sub, obs_mul; /* normalisation: x = ((float)byte - obs_sub) * obs_mul */
  int32_t rnn_type; /* SF_RNN_GRU, or SF_RNN_LSTM (the core of the paper's benchmark model, App.
                       "Model architectures").  A state row ("state_dim" floats below) is
                       h [rnn_dim] for a GRU and [h | c] = 2 * rnn_dim floats for an LSTM. */
  int32_t meas_dim; /* > 0: the "full" architecture (paper, App. "VizDoom experiments"): each row
                       also carries meas_dim fp32 measurements (health, ammunition, ...), which
                       pass n_meas_layers fully connected + ReLU layers of widths meas_hidden[]
                       and are appended to the FC layer's output: the core's input then has
                       fc_dim + meas_hidden[n_meas_layers - 1] features.  0: no such input. */
  int32_t n_meas_layers; /* 1..SF_MAX_MEAS_LAYERS when meas_dim > 0 */
  int32_t meas_hidden[SF_MAX_MEAS_LAYERS];
} sf_policy_config;

/* HOST pointers to fp32 parameters in canonical layouts; read during create only.  Every
 * value must be finite (SF_ERR_ARG otherwise).
 *   conv_w[i]: [cout][cin][k][k], conv_b[i]: [cout].  Residual encoder: per stage
 *              the stage convolution, then each block's two convolutions in order.
 *   fc_w: [fc_dim][flat], flat index = c*(Hf*Wf) + y*Wf + x of the encoder output.
 *   GRU:  rnn_w_ih [3H][core_in], rnn_w_hh [3H][H], rnn_b_ih [3H], rnn_b_hh [3H], with
 *         core_in = fc_dim (+ the last measurement layer's width); gate rows r, z, n:
 *           r = sigmoid(W_ir x + b_ir + W_hr h + b_hr)
 *           z = sigmoid(W_iz x + b_iz + W_hz h + b_hz)
 *           n = tanh   (W_in x + b_in + r * (W_hn h + b_hn))
 *           h_out = (1 - z) * n + z * h,   h = done ? 0 : h_in
 *   LSTM: the same four tensors with 4H rows; gate rows i, f, g, o:
 *           i, f, o = sigmoid(W_i* x + b_i* + W_h* h + b_h*)
 *           g = tanh(W_ig x + b_ig + W_hg h + b_hg)
 *           c_out = f * c + i * g,  h_out = o * tanh(c_out),  (h, c) = done ? 0 : state_in
 *   meas_w[l]: [meas_hidden[l]][width of the previous layer (meas_dim for l = 0)],
 *   meas_b[l]: [meas_hidden[l]]; unused when meas_dim == 0
 *   pi_w: [sum(head_sizes)][H], pi_b: [sum(head_sizes)] (heads concatenated in order)
 *   v_w:  [H], v_b: [1] */
typedef struct {
  const float* conv_w[SF_MAX_CONV_TENSORS];
  const float* conv_b[SF_MAX_CONV_TENSORS];
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
  const float* meas_w[SF_MAX_MEAS_LAYERS];
  const float* meas_b[SF_MAX_MEAS_LAYERS];
} sf_policy_weights;

/* Build a policy on HIP device `hip_device`: validates the description, packs the
 * weights into device layouts and allocates the workspace for max_batch rows.
 * On success *out receives the handle.  Errors: SF_ERR_ARG, SF_ERR_SHAPE,
 * SF_ERR_ARCH, SF_ERR_OOM, SF_ERR_DEVICE; *out is then NULL. */
int sf_policy_create(const sf_policy_config* cfg, const sf_policy_weights* weights,
                     int hip_device, sf_policy** out);

/* Arithmetic of the first convolution (paper, App. "Model architectures": the convolutional
 * encoder reads the pixel observation).  The pixels are bytes, so where the layer has the
 * benchmark shape (8x8, stride 4, no padding, 32 channels, 1/3/4 input planes) it runs as an
 * exact integer contraction on the int8 matrix cores against a fixed-point image of the
 * normalisation-folded filter bank: per output channel one scale and three signed digits of
 * radix 254 (two in a bf16 configuration), i.e. every tap carries the same absolute error,
 * at most 2^-24 (2^-16) of the channel's largest tap.  Unlike floating point this loses
 * relative accuracy on taps much smaller than the largest one.  The library therefore tests
 * each bank when it packs it (create, and again at every weight update): with
 *   E_fix = 128 * sum_k |W'[k] - fixed-point image of W'[k]|   (bound for every frame)
 *   E_ref = sqrt(K) * 2^-24 * 255 * sum_k min(|W'[k]|, median non-zero |W'|)   (fp32;
 *           2^-9 * 255 * sum_k min(...) in a bf16 configuration)
 * the digit planes are used only if E_fix <= E_ref in every channel; otherwise an fp32
 * network runs the layer on the fp32 matrix cores (about three times slower for that
 * launch) and a bf16 network takes the third digit plane.  The decision depends on the
 * parameter values only, never on the batch.  sf_policy_op_pipe tells which arithmetic a
 * launch uses ("i8x3", "i8x2", "f32", "bf16", "f16", "valu"); ..._ratio returns the worst
 * channel's E_fix / E_ref for 2 or 3 planes (0 if the layer has another shape, -1 for a
 * null handle). */
const char* sf_policy_op_pipe(const sf_policy* p, int i); /* static storage; "" if out of range */
/* The kernel family launch i runs, for tests and benchmarks that must know which code path a
 * shape took: one of "generic", "conv1_mfma", "gemm_mfma", "conv1_i8", "conv_bf16",
 * "conv3x3_u8", "conv3x3_patch", "conv3x3_stem", "conv3x3_pool", "stem_pool", "conv_pool_regs", "res_block",
 * "res_stage", "conv_image_bf16", "conv12_fused" for a convolution launch, and "pool", "fc",
 * "meas", "rnn", "heads" for the others.  Static storage; "" if out of range or null. */
const char* sf_policy_op_kernel(const sf_policy* p, int i);
double sf_policy_conv1_fixed_point_ratio(const sf_policy* p, int planes);
/* The same test on a filter bank alone, on the host (no device is touched): conv_w host
 * [32][cin][8][8] fp32, cin 1, 3 or 4; dtype SF_DTYPE_FP32 or SF_DTYPE_BF16 (the taps are
 * first rounded to bf16).  Writes the worst channel's E_fix / E_ref for two and for three
 * digit planes.  Errors: SF_ERR_ARG. */
int sf_conv1_fixed_point_test(const float* conv_w, int32_t cin, float obs_mul, int32_t dtype,
                              double* ratio2, double* ratio3);

/* One step of the policy worker (paper, Sec. 3.1) on B rows, enqueued
 * asynchronously on `hip_stream` (a hipStream_t; NULL = the default stream).
 *   obs        dev  [B][obs_c][obs_h][obs_w] bytes (planar frames), 4-byte aligned
 *   meas       dev  [B][meas_dim] fp32, 4-byte aligned; ignored (may be NULL) when the
 *                   policy has no measurement input
 *   h_in       dev  [B][state_dim] fp32, 16-byte aligned
 *   done       dev  [B] bytes; non-zero = this observation is the first of a new
 *                   episode: the incoming state is zeroed before the GRU cell
 *   seed, step      sampler key and time step.  Category i of head k in row b is
 *                   perturbed with Gumbel noise from word (i mod 4) of
 *                   Philox4x32-10(key = (seed lo, seed hi),
 *                                 counter = (b, step lo, step hi, k << 16 | i / 4)),
 *                   u = ((word >> 9) + 0.5) * 2^-23, g = -log(-log(u)) in fp32;
 *                   the action is the lowest index maximising logit + g.
 *   actions    dev  [B][n_heads] int32
 *   logp       dev  [B] fp32, log-probability of the sampled joint action
 *   value      dev  [B] fp32
 *   h_out      dev  [B][state_dim] fp32, 16-byte aligned; must not overlap h_in
 *   logits_opt dev  [B][sum(head_sizes)] fp32, or NULL if not wanted
 * B == 0 is accepted and does nothing.  Errors: SF_ERR_ARG (null handle or
 * pointer, misaligned pointer), SF_ERR_BATCH, SF_ERR_ALIAS,
 * SF_ERR_DEVICE (a launch failed).  Nothing is enqueued when an error is
 * returned for the arguments. */
int sf_policy_step(sf_policy* p, int32_t B, const uint8_t* obs, const float* meas,
                   const float* h_in, const uint8_t* done, uint64_t seed, uint64_t step,
                   int32_t* actions, float* logp, float* value, float* h_out, float* logits_opt,
                   void* hip_stream);

/* The same step when the batch rows are a subset of a larger population of
 * environments whose recurrent states live in one device table (paper, Sec. 3.3:
 * the components exchange indices into preallocated tensors, never the tensors;
 * Sec. 3.2: with double-buffered sampling the policy worker is given the two
 * halves of a worker's environments in alternation).  Row b stands for
 * environment e = env_ids[b]:
 *   h_table    dev  [n_env][state_dim] fp32, 16-byte aligned.  Row e is read as the
 *                   row's incoming state (zeroed by done[b] as above) and
 *                   overwritten with its new state; rows that no batch row names
 *                   are not touched.
 *   env_ids    dev  [B] int32, 4-byte aligned, distinct, each in [0, n_env).
 *                   The sampler's counter word for row b is e (not b), so what an
 *                   environment draws does not depend on its place in a batch.
 * All other arguments as for sf_policy_step; logits_opt, actions, logp and value
 * are indexed by the batch row b.  The ids are device data and are not checked
 * on the host: a row whose id is outside [0, n_env) is computed from a zero
 * state and its new state is dropped; if two rows name the same environment, the
 * table row ends up with one of their states.  The new states pass through the
 * handle's workspace, so the call is, like sf_policy_step, asynchronous and
 * allocation-free.  Errors: SF_ERR_ARG (null handle or pointer, misaligned
 * pointer, n_env < 1), SF_ERR_BATCH, SF_ERR_DEVICE. */
int sf_policy_step_indexed(sf_policy* p, int32_t B, const uint8_t* obs, const float* meas,
                           float* h_table, int32_t n_env, const int32_t* env_ids, const uint8_t* done,
                           uint64_t seed, uint64_t step, int32_t* actions, float* logp,
                           float* value, float* logits_opt, void* hip_stream);

/* The learner's forward pass over N trajectories of T steps (paper, Sec. 3.1: the learner
 * recomputes the network on the collected trajectories, the recurrent core unrolled over
 * their T steps; hyperparameter table of App. "VizDoom experiments": rollout T = 32, batch of
 * 2048 samples = 64 trajectories).  Its outputs are what sf_appo_loss takes as `logits` and
 * as the first T rows of `values`.  All arrays time-major, on the device:
 *   obs     dev  [T][N][obs_c][obs_h][obs_w] bytes, 4-byte aligned
 *   meas    dev  [T][N][meas_dim] fp32 (NULL without that input)
 *   h0      dev  [N][state_dim] fp32, 16-byte aligned: the state each trajectory started from
 *   done    dev  [T][N] bytes: non-zero at (t, n) = step t of trajectory n begins an episode,
 *                its incoming state is zero
 *   logits  dev  [T][N][sum(head_sizes)] fp32;  value  dev [T][N] fp32
 *   h_seq   dev  [T][N][state_dim] fp32, 16-byte aligned, must not overlap h0: row t is the
 *                state after step t (the last row is the state the trajectories end in)
 * The result is that of T calls of sf_policy_step, time t on rows [t][0..N) with the state
 * rows time t - 1 wrote, except that no action is drawn.  The launches: the encoder and the
 * FC layer once on all T * N frames, the core T times on N rows, the heads once on T * N
 * states; the features pass through the handle's workspace, hence T * N <= max_batch, and
 * N rows of features and of state must be a multiple of 16 bytes.  Asynchronous on
 * hip_stream; allocates nothing.  N == 0 does nothing.  Errors: SF_ERR_ARG (null or
 * misaligned pointer), SF_ERR_BATCH (T < 1, N < 0, T * N > max_batch), SF_ERR_SHAPE (the
 * 16-byte rule), SF_ERR_ALIAS, SF_ERR_DEVICE. */
int sf_policy_unroll(sf_policy* p, int32_t T, int32_t N, const uint8_t* obs, const float* meas,
                     const float* h0, const uint8_t* done, float* logits, float* value,
                     float* h_seq, void* hip_stream);

/* Replace the policy's parameters by new values of the same shapes (paper, Sec. 3.3: after
 * every learner step the policy workers fetch the new parameters; Sec. 3.4: the fresher
 * the sampling policy, the smaller the policy lag).  `weights` as for sf_policy_create:
 * host pointers, read and repacked before the call returns; the packed values then travel
 * to the device as asynchronous copies on `hip_stream`, into the buffers the kernels read.
 * Ordering is the stream's: steps enqueued on that stream before the call use the old
 * parameters, steps enqueued after it the new ones, and no step sees a mixture.  Work on
 * other streams is not ordered against the update.  The first call allocates a page-locked
 * staging area of the size of the packed weights (kept until destroy); a later call first
 * waits for the previous update's copies.  The whole set is packed and checked before the
 * first copy is enqueued: after an error other than SF_ERR_DEVICE the policy still holds its
 * previous parameters.  The kernels are those chosen at create (environment switches are not
 * read again), with one exception: the first convolution's admission test (see
 * sf_policy_op_pipe) is repeated on the new values, and later steps run the arithmetic it
 * selects.  A HIP graph captured before the update keeps the kernel it recorded, which then
 * reads the new bank of its own kind: capture again if the selection changed.
 * Errors: SF_ERR_ARG (null handle or weight pointer), SF_ERR_OOM (staging area),
 * SF_ERR_DEVICE, SF_ERR_SHAPE (internal mismatch). */
int sf_policy_update_weights(sf_policy* p, const sf_policy_weights* weights, void* hip_stream);

/* Floats per recurrent-state row of this policy: rnn_dim (GRU) or 2 * rnn_dim (LSTM). */
int32_t sf_policy_state_dim(const sf_policy* p);

/* Free the workspace and the packed weights.  The caller must have synchronised
 * every stream the handle was stepped on.  NULL is accepted. */
int sf_policy_destroy(sf_policy* p);

/* Text of the last error on this thread (static storage; empty if none). */
const char* sf_last_error(void);

/* Number of floating point operations (2 per multiply-add) of one row of the
 * step for this policy's network, as used by the benchmark's roofline figures. */
int64_t sf_policy_flops_per_row(const sf_policy* p);

/* ---- measurement aids (used by the benchmark; not part of the step) ----------
 * The step is a fixed sequence of kernel launches ("ops": the convolutions, the
 * FC layer, the GRU cell, the heads).  With timing enabled sf_policy_step records
 * a HIP event on its stream before the first and after every launch;
 * sf_policy_last_op_times waits for the last recorded step and writes the
 * duration of each launch in milliseconds to ms_out[0..op_count).  Errors:
 * SF_ERR_ARG (null handle or buffer, n < op_count), SF_ERR_DEVICE (nothing
 * recorded yet). */
int sf_policy_op_count(const sf_policy* p);
const char* sf_policy_op_name(const sf_policy* p, int i); /* static per handle; "" if out of range */
int64_t sf_policy_op_flops_per_row(const sf_policy* p, int i);
int sf_policy_set_op_timing(sf_policy* p, int enable);
int sf_policy_last_op_times(sf_policy* p, float* ms_out /* host */, int n);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both dev pointers
 * 16-byte aligned), asynchronous on hip_stream.  It exists as the known-size
 * reference kernel against which hardware byte counters are scaled when the
 * step's HBM traffic is measured.  Errors: SF_ERR_ARG, SF_ERR_DEVICE. */
int sf_copy_bytes(const void* src, void* dst, int64_t bytes, void* hip_stream);

/* ---- double-buffered stepping -------------------------------------------------
 * A pipeline owns `n_slots` (1 or 2) sets of device buffers for the inputs and
 * outputs of an indexed step on up to slot_batch rows, and three streams of its
 * own: host-to-device copies, compute, device-to-host copies.  While the step of
 * one slot computes, the observations of the other slot cross the bus: this is
 * the policy-worker side of double-buffered sampling (paper, Sec. 3.2), where two
 * groups of environments take turns, one being simulated while the actions of the
 * other are computed.  The steps of the slots run in submission order on the one
 * compute stream (they share the policy's workspace and the state table).
 *
 * sf_pipeline_submit enqueues, for slot `slot`: the copies of obs, meas, done and
 * env_ids to the device, sf_policy_step_indexed on them, and the copies of
 * actions, logp and value back to the host; it returns without waiting.
 *   host_obs      host [B][obs_c][obs_h][obs_w] bytes
 *   host_meas     host [B][meas_dim] fp32; ignored (may be NULL) without a measurement input
 *   host_done     host [B] bytes;  host_env_ids  host [B] int32
 *   h_table       dev  [n_env][state_dim] fp32 (stays on the device)
 *   host_actions  host [B][n_heads] int32; host_logp, host_value  host [B] fp32
 * Host buffers should be page-locked (hipHostMalloc); with pageable memory the
 * copies still work but do not overlap.  They belong to the caller and must stay
 * valid and unmodified (inputs) or unread (outputs) until sf_pipeline_wait(slot)
 * has returned.  A slot that has been submitted must be waited for before it is
 * submitted again (SF_ERR_ARG otherwise).  sf_pipeline_wait blocks the calling
 * thread until the slot's results are in host memory; waiting for an idle slot
 * returns at once.  The policy must outlive the pipeline and must not be stepped
 * by other callers while a slot is in flight.
 * Errors: SF_ERR_ARG (null pointer, bad slot, slot busy, n_slots not 1 or 2),
 * SF_ERR_BATCH (B outside [0, slot_batch], slot_batch outside [1, max_batch]),
 * SF_ERR_OOM, SF_ERR_DEVICE. */
typedef struct sf_pipeline sf_pipeline; /* opaque */
int sf_pipeline_create(sf_policy* policy, int32_t slot_batch, int32_t n_slots, sf_pipeline** out);
int sf_pipeline_submit(sf_pipeline* pl, int32_t slot, int32_t B, const uint8_t* host_obs,
                       const float* host_meas, const uint8_t* host_done,
                       const int32_t* host_env_ids, float* h_table,
                       int32_t n_env, uint64_t seed, uint64_t step, int32_t* host_actions,
                       float* host_logp, float* host_value);
int sf_pipeline_wait(sf_pipeline* pl, int32_t slot);
/* Waits for every slot in flight, then frees buffers, streams and events.  NULL is accepted. */
int sf_pipeline_destroy(sf_pipeline* pl);

/* ---- learner-side loss -------------------------------------------------------
 * The loss of the paper's learner on N trajectories of T steps (Sec. 3.4: V-trace
 * value targets with truncated importance weights, combined with the PPO clipping
 * range; hyperparameter table of App. "VizDoom experiments": rho_bar = c_bar = 1,
 * clipping range [1/1.1, 1.1], entropy coefficient 0.003, critic-loss coefficient
 * 0.5, rollout length 32, 2048 samples per batch), forward values and the gradients
 * with respect to the network's outputs.  The paper cites the two methods without
 * formulas; these are the published ones:
 *   pi = softmax per head of logits[t][n],  logp_pi = sum over heads of log pi(action)
 *   ratio = exp(logp_pi - logp_mu),  rho = min(rho_bar, ratio),  c = min(c_bar, ratio)
 *   g_t = gamma * (1 - done_t),       delta_t = rho_t * (r_t + g_t V_{t+1} - V_t)
 *   vs_t - V_t = delta_t + g_t c_t (vs_{t+1} - V_{t+1}),  vs_T = V_T
 *   adv_t = r_t + g_t vs_{t+1} - V_t
 *   L_pi = -mean min(ratio adv, clamp(ratio, 1/clip, clip) adv)
 *   L_v = critic_coef * mean (V_t - vs_t)^2,   L_ent = -entropy_coef * mean sum_heads entropy
 * with means over the T*N samples; the gradients treat vs and adv as constants.
 * All arrays are device memory, time-major, 4-byte aligned:
 *   logits   [T][N][sum(head_sizes)] fp32     actions [T][N][n_heads] int32 (an action
 *                                             outside its head is clamped into it)
 *   logp_mu  [T][N] fp32: joint log-probability under the behaviour policy (the logp
 *                         output of sf_policy_step when the sample was taken)
 *   values   [T+1][N] fp32, row T = bootstrap value;  rewards [T][N] fp32;  dones [T][N] bytes
 *   vs, adv  [T][N] fp32 out;  loss [4] fp32 out = {L_pi, L_v, L_ent, their sum}
 *   dlogits_opt [T][N][sum(head_sizes)], dvalues_opt [T][N] (d/dV_t of L_v) fp32 out, or NULL
 *   workspace   sf_appo_loss_workspace_bytes(cfg) bytes (16 N + 16), owned by the caller
 * Asynchronous on hip_stream, allocation-free, and bitwise reproducible (the partial sums
 * are added in a fixed order).  Errors: SF_ERR_ARG (null or misaligned pointer, struct_size),
 * SF_ERR_SHAPE (sizes or hyperparameters out of range), SF_ERR_DEVICE. */
typedef struct {
  uint32_t struct_size; /* sizeof(sf_loss_config) */
  int32_t T, N, n_heads;
  int32_t head_sizes[SF_MAX_HEADS];
  float gamma, rho_bar, c_bar, clip, critic_coef, entropy_coef;
} sf_loss_config;
int64_t sf_appo_loss_workspace_bytes(const sf_loss_config* cfg); /* -1 on a bad configuration */
int sf_appo_loss(const sf_loss_config* cfg, const float* logits, const int32_t* actions,
                 const float* logp_mu, const float* values, const float* rewards,
                 const uint8_t* dones, float* vs, float* adv, float* loss, float* dlogits_opt,
                 float* dvalues_opt, void* workspace, void* hip_stream);


/* The same loss for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid allocation.  The
 * per-trajectory partial sums (N x 16 bytes) live in an array inside the library's device
 * image, 256 KiB per GPU for as long as the process runs, so N is limited to
 * sf_appo_loss_static_max_trajectories() = 16384; a larger N is refused with SF_ERR_SHAPE.  The
 * call allocates and frees nothing, runs on the current HIP device, and is otherwise
 * sf_appo_loss (same kernels, same bits).  All calls on one GPU share the one array, which
 * keeps the last call's contents (every slot a call reads is written by that call first): two
 * calls that overlap on one GPU, on different streams or from different threads, race; calls
 * on one stream are safe.  Errors: as sf_appo_loss, plus SF_ERR_SHAPE for N beyond the limit
 * and SF_ERR_DEVICE if the array's address cannot be obtained. */
int32_t sf_appo_loss_static_max_trajectories(void);
int sf_appo_loss_static(const sf_loss_config* cfg, const float* logits, const int32_t* actions,
                        const float* logp_mu, const float* values, const float* rewards,
                        const uint8_t* dones, float* vs, float* adv, float* loss, float* dlogits_opt,
                        float* dvalues_opt, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif

/*
 * CPU oracle for the policy worker's batched actor-critic step: test
 * infrastructure only (see sf_oracle.h for scope, arithmetic and pins).
 * Plain C, direct loops, fp64 activations.  Build:
 *   gcc -O2 -std=c11 -ffp-contract=off -fopenmp -fPIC -shared sf_oracle.c -lm
 */
#include "sf_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* Encoder pieces (paper, App. "Model architectures": conv layers, then FC).  */

int ref_conv2d(const double* in, int C, int H, int W, const float* w, const float* bias, int O,
               int k, int s, int pad, int relu, double* out) {
  if (s < 1 || k < 1 || pad < 0) return -1;
  int Ho = (H + 2 * pad - k) / s + 1;
  int Wo = (W + 2 * pad - k) / s + 1;
  if (H + 2 * pad < k || W + 2 * pad < k || Ho < 1 || Wo < 1) return -1;
  for (int o = 0; o < O; ++o)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        double acc = (double)bias[o];
        for (int c = 0; c < C; ++c)
          for (int p = 0; p < k; ++p) {
            int y = i * s + p - pad;
            if (y < 0 || y >= H) continue;
            for (int q = 0; q < k; ++q) {
              int x = j * s + q - pad;
              if (x < 0 || x >= W) continue;
              acc += (double)w[((o * C + c) * k + p) * k + q] * in[(c * H + y) * W + x];
            }
          }
        if (relu && acc < 0.0) acc = 0.0;
        out[(o * Ho + i) * Wo + j] = acc;
      }
  return 0;
}

void ref_maxpool3x3s2p1(const double* in, int C, int H, int W, double* out) {
  int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  for (int c = 0; c < C; ++c)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        double m = -INFINITY;
        for (int y = 2 * i - 1; y <= 2 * i + 1; ++y) {
          if (y < 0 || y >= H) continue;
          for (int x = 2 * j - 1; x <= 2 * j + 1; ++x) {
            if (x < 0 || x >= W) continue;
            double v = in[(c * H + y) * W + x];
            if (v > m) m = v;
          }
        }
        out[(c * Ho + i) * Wo + j] = m;
      }
}

void ref_linear(const double* in, int n_in, const float* w, const float* bias, int n_out,
                int relu, double* out) {
  for (int o = 0; o < n_out; ++o) {
    double acc = (double)bias[o];
    for (int i = 0; i < n_in; ++i) acc += (double)w[(size_t)o * n_in + i] * in[i];
    if (relu && acc < 0.0) acc = 0.0;
    out[o] = acc;
  }
}

static double sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }

void ref_gru_cell(const double* x, int n_in, const double* h, int H, const float* w_ih,
                  const float* w_hh, const float* b_ih, const float* b_hh, double* h_new) {
  double* gi = (double*)malloc(sizeof(double) * 3 * (size_t)H);
  double* gh = (double*)malloc(sizeof(double) * 3 * (size_t)H);
  ref_linear(x, n_in, w_ih, b_ih, 3 * H, 0, gi); /* W_i* x + b_i* for r, z, n */
  ref_linear(h, H, w_hh, b_hh, 3 * H, 0, gh);    /* W_h* h + b_h* for r, z, n */
  for (int j = 0; j < H; ++j) {
    double r = sigmoid(gi[j] + gh[j]);
    double z = sigmoid(gi[H + j] + gh[H + j]);
    double n = tanh(gi[2 * H + j] + r * gh[2 * H + j]);
    h_new[j] = (1.0 - z) * n + z * h[j];
  }
  free(gi);
  free(gh);
}

void ref_lstm_cell(const double* x, int n_in, const double* h, const double* c, int H,
                   const float* w_ih, const float* w_hh, const float* b_ih, const float* b_hh,
                   double* h_new, double* c_new) {
  double* gi = (double*)malloc(sizeof(double) * 4 * (size_t)H);
  double* gh = (double*)malloc(sizeof(double) * 4 * (size_t)H);
  ref_linear(x, n_in, w_ih, b_ih, 4 * H, 0, gi); /* W_i* x + b_i* for i, f, g, o */
  ref_linear(h, H, w_hh, b_hh, 4 * H, 0, gh);    /* W_h* h + b_h* for i, f, g, o */
  for (int j = 0; j < H; ++j) {
    double ig = sigmoid(gi[j] + gh[j]);
    double fg = sigmoid(gi[H + j] + gh[H + j]);
    double gg = tanh(gi[2 * H + j] + gh[2 * H + j]);
    double og = sigmoid(gi[3 * H + j] + gh[3 * H + j]);
    c_new[j] = fg * c[j] + ig * gg;
    h_new[j] = og * tanh(c_new[j]);
  }
  free(gi);
  free(gh);
}

static void relu_copy(const double* in, size_t n, double* out) {
  for (size_t i = 0; i < n; ++i) out[i] = in[i] > 0.0 ? in[i] : 0.0;
}

int ref_resnet_encoder(const ref_net* net, const ref_params* p, const double* x, double* out,
                       int* hf, int* wf) {
  int C = net->obs_c, H = net->obs_h, W = net->obs_w;
  int maxc = C;
  for (int s = 0; s < net->n_stage; ++s)
    if (net->stage_ch[s] > maxc) maxc = net->stage_ch[s];
  size_t cap = (size_t)maxc * H * W;
  double* cur = (double*)malloc(sizeof(double) * cap);
  double* t0 = (double*)malloc(sizeof(double) * cap);
  double* t1 = (double*)malloc(sizeof(double) * cap);
  memcpy(cur, x, sizeof(double) * (size_t)C * H * W);
  int ti = 0; /* index into conv_w / conv_b */
  for (int s = 0; s < net->n_stage; ++s) {
    int O = net->stage_ch[s];
    ref_conv2d(cur, C, H, W, p->conv_w[ti], p->conv_b[ti], O, 3, 1, 1, 0, t0);
    ++ti;
    ref_maxpool3x3s2p1(t0, O, H, W, cur);
    C = O;
    H = (H - 1) / 2 + 1;
    W = (W - 1) / 2 + 1;
    size_t n = (size_t)C * H * W;
    for (int b = 0; b < net->blocks_per_stage; ++b) {
      relu_copy(cur, n, t0);
      ref_conv2d(t0, C, H, W, p->conv_w[ti], p->conv_b[ti], C, 3, 1, 1, 1, t1); /* relu(conv_a) */
      ++ti;
      ref_conv2d(t1, C, H, W, p->conv_w[ti], p->conv_b[ti], C, 3, 1, 1, 0, t0);
      ++ti;
      for (size_t i = 0; i < n; ++i) cur[i] += t0[i];
    }
  }
  relu_copy(cur, (size_t)C * H * W, out);
  *hf = H;
  *wf = W;
  free(cur);
  free(t0);
  free(t1);
  return 0;
}

/* ------------------------------------------------------------------------ */
/* Sampler: counter-based Philox4x32-10 -> uniform -> Gumbel -> argmax.       */

void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0;
    c1 = n1;
    c2 = n2;
    c3 = n3;
    k0 += 0x9E3779B9u; /* key schedule: golden-ratio and sqrt(3)-1 constants */
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

float ref_bits_to_uniform(uint32_t w) {
  return ((float)(w >> 9) + 0.5f) * 0x1.0p-23f;
}

void ref_bits_to_uniform_many(const uint32_t* w, int64_t n, float* u) {
  for (int64_t i = 0; i < n; ++i) u[i] = ref_bits_to_uniform(w[i]);
}

float ref_gumbel(float u) {
  float inner = -logf(u);
  return -logf(inner);
}

void ref_sampler_words(uint64_t seed, uint32_t env, uint64_t step, uint32_t head, uint32_t block,
                       uint32_t out[4]) {
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t ctr[4] = {env, (uint32_t)step, (uint32_t)(step >> 32), (head << 16) | block};
  ref_philox4x32_10(ctr, key, out);
}

void ref_log_softmax(const float* logits, int A, double* out) {
  double m = (double)logits[0];
  for (int i = 1; i < A; ++i)
    if ((double)logits[i] > m) m = (double)logits[i];
  double s = 0.0;
  for (int i = 0; i < A; ++i) s += exp((double)logits[i] - m);
  double lse = m + log(s);
  for (int i = 0; i < A; ++i) out[i] = (double)logits[i] - lse;
}

void ref_head_sample(const float* logits, int A, uint64_t seed, uint32_t env, uint64_t step,
                     uint32_t head, const float* g_override, int32_t* action, double* logp,
                     float* margin) {
  float best = -INFINITY, second = -INFINITY;
  int arg = 0;
  uint32_t words[4] = {0, 0, 0, 0};
  for (int i = 0; i < A; ++i) {
    float g;
    if (g_override) {
      g = g_override[i];
    } else {
      if ((i & 3) == 0) ref_sampler_words(seed, env, step, head, (uint32_t)(i >> 2), words);
      g = ref_gumbel(ref_bits_to_uniform(words[i & 3]));
    }
    float pert = logits[i] + g;
    if (i == 0) {
      best = pert;
      arg = 0;
    } else if (pert > best) { /* strict: ties keep the lowest index */
      second = best;
      best = pert;
      arg = i;
    } else if (pert > second) {
      second = pert;
    }
  }
  double* ls = (double*)malloc(sizeof(double) * (size_t)A);
  ref_log_softmax(logits, A, ls);
  *action = arg;
  *logp = ls[arg];
  if (margin) *margin = (A > 1) ? best - second : INFINITY;
  free(ls);
}

void ref_head_histogram(const float* logits, int A, uint64_t seed, uint32_t head, int64_t n,
                        uint32_t n_env, uint64_t step0, int64_t* counts) {
  for (int i = 0; i < A; ++i) counts[i] = 0;
  for (int64_t d = 0; d < n; ++d) {
    int32_t a;
    double lp;
    ref_head_sample(logits, A, seed, (uint32_t)(d % n_env), step0 + (uint64_t)(d / n_env), head,
                    NULL, &a, &lp, NULL);
    counts[a] += 1;
  }
}

/* ------------------------------------------------------------------------ */
/* The whole step (paper, Sec. 3.1: (x_t, h_t) -> mu, h_{t+1}; a_t ~ mu).     */

static int encoder_shape(const ref_net* net, int* Cf, int* Hf, int* Wf) {
  int C = net->obs_c, H = net->obs_h, W = net->obs_w;
  if (C < 1 || H < 1 || W < 1) return -1;
  if (net->encoder == 0) {
    if (net->n_conv < 1 || net->n_conv > REF_MAX_CONV) return -1;
    for (int l = 0; l < net->n_conv; ++l) {
      int k = net->conv_k[l], s = net->conv_stride[l], pad = net->conv_pad[l];
      if (k < 1 || s < 1 || pad < 0 || H + 2 * pad < k || W + 2 * pad < k) return -1;
      H = (H + 2 * pad - k) / s + 1;
      W = (W + 2 * pad - k) / s + 1;
      C = net->conv_cout[l];
      if (C < 1) return -1;
    }
  } else if (net->encoder == 1) {
    if (net->n_stage < 1 || net->n_stage > REF_MAX_STAGE || net->blocks_per_stage < 0) return -1;
    if (net->n_stage * (1 + 2 * net->blocks_per_stage) > REF_MAX_CONV_TENSORS) return -1;
    for (int s = 0; s < net->n_stage; ++s) {
      C = net->stage_ch[s];
      if (C < 1) return -1;
      H = (H - 1) / 2 + 1;
      W = (W - 1) / 2 + 1;
    }
  } else {
    return -1;
  }
  *Cf = C;
  *Hf = H;
  *Wf = W;
  return 0;
}

int64_t ref_flat_size(const ref_net* net) {
  int C, H, W;
  if (encoder_shape(net, &C, &H, &W)) return -1;
  return (int64_t)C * H * W;
}

int ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Row b of the batch.  env is the sampler's counter word for this row; h_in_row and
 * h_out_row are this row's incoming and outgoing state (rnn_dim floats each). */
static void step_row(const ref_net* net, const ref_params* p, int32_t b, uint32_t env,
                     const uint8_t* obs, const float* meas, const float* h_in_row,
                     const uint8_t* done, uint64_t seed,
                     uint64_t step, int32_t* actions, float* logp, float* value, float* h_out_row,
                     float* logits_opt, float* margin_opt) {
  const int C = net->obs_c, H = net->obs_h, W = net->obs_w, Hd = net->rnn_dim;
  size_t n_obs = (size_t)C * H * W;

  /* normalised observation (reading: affine map of the byte) */
  double* x = (double*)malloc(sizeof(double) * n_obs);
  const uint8_t* o = obs + (size_t)b * n_obs;
  for (size_t i = 0; i < n_obs; ++i)
    x[i] = ((double)o[i] - (double)net->obs_sub) * (double)net->obs_mul;

  /* encoder */
  int Cf, Hf, Wf;
  encoder_shape(net, &Cf, &Hf, &Wf);
  size_t flat = (size_t)Cf * Hf * Wf;
  double* enc;
  if (net->encoder == 0) {
    double* cur = x;
    int c = C, h = H, w = W;
    for (int l = 0; l < net->n_conv; ++l) {
      int k = net->conv_k[l], s = net->conv_stride[l], pad = net->conv_pad[l];
      int ho = (h + 2 * pad - k) / s + 1, wo = (w + 2 * pad - k) / s + 1;
      double* nxt = (double*)malloc(sizeof(double) * (size_t)net->conv_cout[l] * ho * wo);
      ref_conv2d(cur, c, h, w, p->conv_w[l], p->conv_b[l], net->conv_cout[l], k, s, pad, 1, nxt);
      free(cur);
      cur = nxt;
      c = net->conv_cout[l];
      h = ho;
      w = wo;
    }
    enc = cur; /* [Cf][Hf][Wf], flattened in this (channel-major) order */
  } else {
    enc = (double*)malloc(sizeof(double) * flat);
    int hf, wf;
    ref_resnet_encoder(net, p, x, enc, &hf, &wf);
    free(x);
  }

  /* fully connected layer + ReLU */
  double* f = (double*)malloc(sizeof(double) * (size_t)net->fc_dim);
  ref_linear(enc, (int)flat, p->fc_w, p->fc_b, net->fc_dim, 1, f);

  /* full architecture: the low-dimensional measurement vector goes through its own
   * fully connected layers (+ReLU) and is appended to the encoder's features */
  int n_core_in = net->fc_dim;
  double* core_in = f;
  if (net->meas_dim > 0) {
    int n_cur = net->meas_dim;
    double* cur = (double*)malloc(sizeof(double) * (size_t)n_cur);
    for (int i = 0; i < n_cur; ++i) cur[i] = (double)meas[(size_t)b * net->meas_dim + i];
    for (int l = 0; l < net->n_meas_layers; ++l) {
      double* nxt = (double*)malloc(sizeof(double) * (size_t)net->meas_hidden[l]);
      ref_linear(cur, n_cur, p->meas_w[l], p->meas_b[l], net->meas_hidden[l], 1, nxt);
      free(cur);
      cur = nxt;
      n_cur = net->meas_hidden[l];
    }
    n_core_in = net->fc_dim + n_cur;
    core_in = (double*)malloc(sizeof(double) * (size_t)n_core_in);
    memcpy(core_in, f, sizeof(double) * (size_t)net->fc_dim);
    memcpy(core_in + net->fc_dim, cur, sizeof(double) * (size_t)n_cur);
    free(cur);
  }

  /* recurrent core with the episode-boundary reset applied to the INCOMING state; an
   * LSTM's state row is [h | c] and both halves are reset */
  const int lstm = net->rnn_type == 1;
  double* h = (double*)malloc(sizeof(double) * (size_t)Hd * 2);
  double* hn = (double*)malloc(sizeof(double) * (size_t)Hd * 2);
  for (int j = 0; j < (lstm ? 2 * Hd : Hd); ++j) h[j] = done[b] ? 0.0 : (double)h_in_row[j];
  if (lstm)
    ref_lstm_cell(core_in, n_core_in, h, h + Hd, Hd, p->rnn_w_ih, p->rnn_w_hh, p->rnn_b_ih,
                  p->rnn_b_hh, hn, hn + Hd);
  else
    ref_gru_cell(core_in, n_core_in, h, Hd, p->rnn_w_ih, p->rnn_w_hh, p->rnn_b_ih, p->rnn_b_hh, hn);
  for (int j = 0; j < (lstm ? 2 * Hd : Hd); ++j) h_out_row[j] = (float)hn[j];
  if (core_in != f) free(core_in);

  /* heads: action logits (all heads concatenated) and the baseline */
  int sumA = 0;
  for (int k = 0; k < net->n_heads; ++k) sumA += net->head_sizes[k];
  double* ld = (double*)malloc(sizeof(double) * (size_t)sumA);
  float* lf = (float*)malloc(sizeof(float) * (size_t)sumA);
  ref_linear(hn, Hd, p->pi_w, p->pi_b, sumA, 0, ld);
  for (int i = 0; i < sumA; ++i) lf[i] = (float)ld[i];
  double v;
  ref_linear(hn, Hd, p->v_w, p->v_b, 1, 0, &v);
  value[b] = (float)v;
  if (logits_opt) memcpy(logits_opt + (size_t)b * sumA, lf, sizeof(float) * (size_t)sumA);

  /* independent categorical heads: sample each, add the log-probabilities */
  double lp_sum = 0.0;
  int off = 0;
  for (int k = 0; k < net->n_heads; ++k) {
    int32_t a;
    double lp;
    float mg;
    ref_head_sample(lf + off, net->head_sizes[k], seed, env, step, (uint32_t)k, NULL, &a,
                    &lp, &mg);
    actions[(size_t)b * net->n_heads + k] = a;
    if (margin_opt) margin_opt[(size_t)b * net->n_heads + k] = mg;
    lp_sum += lp;
    off += net->head_sizes[k];
  }
  logp[b] = (float)lp_sum;

  free(enc);
  free(f);
  free(h);
  free(hn);
  free(ld);
  free(lf);
}

static int check_net(const ref_net* net) {
  int C, H, W;
  if (encoder_shape(net, &C, &H, &W)) return -1;
  if (net->fc_dim < 1 || net->rnn_dim < 1 || net->n_heads < 1 || net->n_heads > REF_MAX_HEADS)
    return -1;
  for (int k = 0; k < net->n_heads; ++k)
    if (net->head_sizes[k] < 1) return -1;
  if (net->rnn_type != 0 && net->rnn_type != 1) return -1;
  if (net->meas_dim < 0) return -1;
  if (net->meas_dim > 0) {
    if (net->n_meas_layers < 1 || net->n_meas_layers > REF_MAX_MEAS_LAYERS) return -1;
    for (int l = 0; l < net->n_meas_layers; ++l)
      if (net->meas_hidden[l] < 1) return -1;
  }
  return 0;
}

int ref_state_dim(const ref_net* net) { return net->rnn_dim * (net->rnn_type == 1 ? 2 : 1); }

int ref_policy_step(const ref_net* net, const ref_params* p, int32_t B, const uint8_t* obs,
                    const float* meas, const float* h_in, const uint8_t* done, uint64_t seed,
                    uint64_t step, int32_t* actions, float* logp, float* value, float* h_out,
                    float* logits_opt, float* margin_opt) {
  if (check_net(net) || B < 0) return -1;
  if (net->meas_dim > 0 && B > 0 && !meas) return -1;
  const size_t Sd = (size_t)ref_state_dim(net);
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t b = 0; b < B; ++b)
    step_row(net, p, b, (uint32_t)b, obs, meas, h_in + (size_t)b * Sd, done, seed, step, actions,
             logp, value, h_out + (size_t)b * Sd, logits_opt, margin_opt);
  return 0;
}

int ref_policy_step_indexed(const ref_net* net, const ref_params* p, int32_t B, const uint8_t* obs,
                            const float* meas, float* h_table, int32_t n_env, const int32_t* env_ids,
                            const uint8_t* done, uint64_t seed, uint64_t step, int32_t* actions,
                            float* logp, float* value, float* logits_opt, float* margin_opt) {
  if (check_net(net) || B < 0 || n_env < 0) return -1;
  if (net->meas_dim > 0 && B > 0 && !meas) return -1;
  /* every row names its own environment */
  unsigned char* seen = (unsigned char*)calloc((size_t)n_env + 1, 1);
  int bad = 0;
  for (int32_t b = 0; b < B; ++b) {
    if (env_ids[b] < 0 || env_ids[b] >= n_env || seen[env_ids[b]]) {
      bad = 1;
      break;
    }
    seen[env_ids[b]] = 1;
  }
  free(seen);
  if (bad) return -2;
  const size_t Hd = (size_t)ref_state_dim(net);
  /* all rows read the table before any row writes it */
  float* h_new = (float*)malloc(sizeof(float) * (size_t)(B > 0 ? B : 1) * Hd);
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t b = 0; b < B; ++b)
    step_row(net, p, b, (uint32_t)env_ids[b], obs, meas, h_table + (size_t)env_ids[b] * Hd, done, seed,
             step, actions, logp, value, h_new + (size_t)b * Hd, logits_opt, margin_opt);
  for (int32_t b = 0; b < B; ++b)
    memcpy(h_table + (size_t)env_ids[b] * Hd, h_new + (size_t)b * Hd, sizeof(float) * Hd);
  free(h_new);
  return 0;
}

/* ---- learner's forward pass over trajectories -------------------------------- */

int ref_policy_unroll(const ref_net* net, const ref_params* p, int32_t T, int32_t N,
                      const uint8_t* obs, const float* meas, const float* h0, const uint8_t* done,
                      float* logits, float* value, float* h_seq) {
  if (check_net(net) || T < 1 || N < 0) return -1;
  if (net->meas_dim > 0 && N > 0 && !meas) return -1;
  const size_t Sd = (size_t)ref_state_dim(net);
  const size_t frame = (size_t)net->obs_c * net->obs_h * net->obs_w;
  size_t sumA = 0;
  for (int k = 0; k < net->n_heads; ++k) sumA += (size_t)net->head_sizes[k];
  /* the step draws actions as well: they are not part of this pass and are dropped */
  int32_t* actions = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1) * net->n_heads);
  float* logp = (float*)malloc(sizeof(float) * (size_t)(N > 0 ? N : 1));
  int rc = 0;
  for (int32_t t = 0; t < T && rc == 0; ++t) {
    const size_t r = (size_t)t * N; /* first row of time t */
    const float* h_prev = t == 0 ? h0 : h_seq + (r - N) * Sd;
    rc = ref_policy_step(net, p, N, obs + r * frame, meas ? meas + r * net->meas_dim : NULL, h_prev,
                         done + r, 0, (uint64_t)t, actions, logp, value + r, h_seq + r * Sd,
                         logits + r * sumA, NULL);
  }
  free(actions);
  free(logp);
  return rc;
}

/* ---- learner-side loss ----------------------------------------------------- */

int ref_appo_loss(const ref_loss_cfg* cfg, const float* logits, const int32_t* actions,
                  const float* logp_mu, const float* values, const float* rewards,
                  const uint8_t* dones, double* vs, double* adv, double* loss, double* dlogits,
                  double* dvalues) {
  const int T = cfg->T, N = cfg->N, nh = cfg->n_heads;
  if (T < 1 || N < 1 || nh < 1 || nh > REF_MAX_HEADS || !(cfg->clip >= 1.0f)) return -1;
  int sumA = 0;
  for (int k = 0; k < nh; ++k) {
    if (cfg->head_sizes[k] < 1) return -1;
    sumA += cfg->head_sizes[k];
  }
  const size_t M = (size_t)T * N;
  for (size_t s = 0; s < M; ++s)
    for (int k = 0; k < nh; ++k)
      if (actions[s * nh + k] < 0 || actions[s * nh + k] >= cfg->head_sizes[k]) return -1;

  double* ratio = (double*)malloc(sizeof(double) * M);
  double* ent = (double*)malloc(sizeof(double) * M);
  double* lsm = (double*)malloc(sizeof(double) * M * (size_t)sumA); /* log softmax per head */
  for (size_t s = 0; s < M; ++s) {
    double lp = 0.0, h = 0.0;
    int off = 0;
    for (int k = 0; k < nh; ++k) {
      const int A = cfg->head_sizes[k];
      double* ls = lsm + s * sumA + off;
      ref_log_softmax(logits + s * sumA + off, A, ls);
      lp += ls[actions[s * nh + k]];
      for (int i = 0; i < A; ++i) h -= exp(ls[i]) * ls[i];
      off += A;
    }
    ratio[s] = exp(lp - (double)logp_mu[s]);
    ent[s] = h;
  }

  /* V-trace targets by their defining sum, then the advantages */
  const double gam = cfg->gamma;
  for (int n = 0; n < N; ++n) {
    for (int t = 0; t < T; ++t) {
      double acc = 0.0, prod = 1.0;
      for (int k = t; k < T; ++k) {
        const size_t s = (size_t)k * N + n;
        const double g = dones[s] ? 0.0 : gam;
        const double rho = ratio[s] < cfg->rho_bar ? ratio[s] : (double)cfg->rho_bar;
        const double c = ratio[s] < cfg->c_bar ? ratio[s] : (double)cfg->c_bar;
        const double delta = rho * ((double)rewards[s] + g * (double)values[s + N] - (double)values[s]);
        acc += prod * delta;
        prod *= g * c;
      }
      vs[(size_t)t * N + n] = (double)values[(size_t)t * N + n] + acc;
    }
    for (int t = 0; t < T; ++t) {
      const size_t s = (size_t)t * N + n;
      const double g = dones[s] ? 0.0 : gam;
      const double vnext = t + 1 < T ? vs[s + N] : (double)values[(size_t)T * N + n];
      adv[s] = (double)rewards[s] + g * vnext - (double)values[s];
    }
  }

  const double lo = 1.0 / (double)cfg->clip, hi = (double)cfg->clip;
  double l_pi = 0.0, l_v = 0.0, l_h = 0.0;
  for (size_t s = 0; s < M; ++s) {
    const double rc = ratio[s] < lo ? lo : (ratio[s] > hi ? hi : ratio[s]);
    const double a = ratio[s] * adv[s], b = rc * adv[s];
    l_pi -= a < b ? a : b;
    const double dv = (double)values[s] - vs[s];
    l_v += dv * dv;
    l_h -= ent[s];
  }
  loss[0] = l_pi / (double)M;
  loss[1] = (double)cfg->critic_coef * l_v / (double)M;
  loss[2] = (double)cfg->entropy_coef * l_h / (double)M;
  loss[3] = loss[0] + loss[1] + loss[2];

  if (dvalues)
    for (size_t s = 0; s < M; ++s)
      dvalues[s] = 2.0 * (double)cfg->critic_coef * ((double)values[s] - vs[s]) / (double)M;
  if (dlogits)
    for (size_t s = 0; s < M; ++s) {
      /* the surrogate follows the unclipped branch where it is the smaller one (ties: the
       * unclipped branch, whose slope the clamped one shares inside the range) */
      const double rc = ratio[s] < lo ? lo : (ratio[s] > hi ? hi : ratio[s]);
      const int unclipped = ratio[s] * adv[s] <= rc * adv[s];
      const double dlp = unclipped ? -adv[s] * ratio[s] / (double)M : 0.0; /* d L_pi / d logp_pi */
      int off = 0;
      for (int k = 0; k < nh; ++k) {
        const int A = cfg->head_sizes[k];
        const double* ls = lsm + s * sumA + off;
        double hk = 0.0;
        for (int i = 0; i < A; ++i) hk -= exp(ls[i]) * ls[i];
        for (int i = 0; i < A; ++i) {
          const double p = exp(ls[i]);
          const double dpol = dlp * ((i == actions[s * nh + k] ? 1.0 : 0.0) - p);
          const double dent = (double)cfg->entropy_coef / (double)M * p * (ls[i] + hk);
          dlogits[s * sumA + off + i] = dpol + dent;
        }
        off += A;
      }
    }
  free(ratio);
  free(ent);
  free(lsm);
  return 0;
}

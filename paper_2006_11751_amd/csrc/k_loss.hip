// Learner-side loss on a batch of trajectories (paper, Sec. 3.4: V-trace targets combined
// with PPO clipping; hyperparameter table of App. "VizDoom experiments"), forward values and
// the gradients with respect to the logits and the values.
//
//   ratio   = exp(logp_pi - logp_mu),  rho = min(rho_bar, ratio),  c = min(c_bar, ratio)
//   g_t     = gamma * (1 - done_t),    delta_t = rho_t * (r_t + g_t V_{t+1} - V_t)
//   vs_t - V_t = delta_t + g_t c_t (vs_{t+1} - V_{t+1}),   vs_T = V_T          (V-trace)
//   adv_t   = r_t + g_t vs_{t+1} - V_t
//   L_pi = -mean min(ratio adv, clamp(ratio, 1/clip, clip) adv),  L_v = c_v mean (V - vs)^2,
//   L_ent = -c_H mean entropy
//
// One 64-lane wavefront per trajectory, one lane per time step.  A lane first reduces its
// sample's logits to the joint log-probability and the entropy; the backward recursion over
// time then runs across the lanes of the wave (the 64 coefficient pairs are broadcast one
// by one, last step first); trajectories longer than 64 steps are walked in 64-step chunks
// from the end, carrying the recursion's value.  The lane then writes targets, advantages
// and gradients for its sample, and the wave its three partial sums.  A second, single-wave
// launch adds the per-trajectory partial sums in a fixed order, so the result does not
// depend on scheduling.
#include <math.h>

#include <mutex>

#include "sf_internal.h"

namespace sf {

namespace {

constexpr int kWave = 64;
constexpr int kTrajPerBlock = 4;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

struct LossArgs {
  const float* logits;    // [T][N][sumA]
  const int32_t* actions; // [T][N][n_heads]
  const float* logp_mu;   // [T][N]
  const float* values;    // [T+1][N]
  const float* rewards;   // [T][N]
  const uint8_t* dones;   // [T][N]
  float* vs;              // [T][N]
  float* adv;             // [T][N]
  float* dlogits;         // [T][N][sumA] or null
  float* dvalues;         // [T][N] or null
  float* partials;        // [N][4]
  int T, N, n_heads, sumA;
  int head_sizes[SF_MAX_HEADS];
  float gamma, rho_bar, c_bar, clip, critic_coef, entropy_coef;
};

__global__ __launch_bounds__(kWave* kTrajPerBlock) void appo_traj_kernel(LossArgs g) {
  const int lane = threadIdx.x % kWave;
  const int n = blockIdx.x * kTrajPerBlock + threadIdx.x / kWave;
  if (n >= g.N) return;  // whole wave leaves together; no block-level barrier below
  const float inv_m = 1.0f / ((float)g.T * (float)g.N);
  const float lo = 1.0f / g.clip, hi = g.clip;
  float sum_pi = 0.0f, sum_v = 0.0f, sum_ent = 0.0f;
  float carry = 0.0f;  // vs - V at the first step of the chunk after this one (0 at t = T)
  const int n_chunks = (g.T + kWave - 1) / kWave;
  for (int ch = n_chunks - 1; ch >= 0; --ch) {
    const int t = ch * kWave + lane;
    const bool live = t < g.T;
    const size_t s = (size_t)(live ? t : g.T - 1) * g.N + n;  // idle lanes re-read the last step
    // joint log-probability of the taken action and entropy, head by head
    float logp = 0.0f, ent = 0.0f;
    {
      const float* l = g.logits + s * g.sumA;
      for (int k = 0; k < g.n_heads; ++k) {
        const int A = g.head_sizes[k];
        float mx = -INFINITY;
        for (int i = 0; i < A; ++i) mx = fmaxf(mx, l[i]);
        float se = 0.0f;
        for (int i = 0; i < A; ++i) se += expf(l[i] - mx);
        const float lse = mx + logf(se);
        float hk = 0.0f;
        for (int i = 0; i < A; ++i) {
          const float ls = l[i] - lse;
          hk -= expf(ls) * ls;
        }
        const int a = min(max(g.actions[s * g.n_heads + k], 0), A - 1);
        logp += l[a] - lse;
        ent += hk;
        l += A;
      }
    }
    const float v = g.values[s], vn = g.values[s + g.N], r = g.rewards[s];
    const float gm = g.dones[s] ? 0.0f : g.gamma;
    const float ratio = expf(logp - g.logp_mu[s]);
    const float rho = fminf(g.rho_bar, ratio), c = fminf(g.c_bar, ratio);
    // idle lanes (past the last step) sit at the start of the backward scan: they pass 0 on
    const float delta = live ? rho * (r + gm * vn - v) : 0.0f;
    const float gc = live ? gm * c : 0.0f;
    float x = carry, mine = 0.0f;
    for (int l = kWave - 1; l >= 0; --l) {
      x = __shfl(delta, l, kWave) + __shfl(gc, l, kWave) * x;
      if (lane == l) mine = x;
    }
    // vs_{t+1} - V_{t+1}: the next lane's value, or the later chunk's first one
    float next = __shfl_down(mine, 1, kWave);
    if (lane == kWave - 1) next = carry;
    carry = __shfl(mine, 0, kWave);
    if (live) {
      const float vs = v + mine;
      const float adv = r + gm * (vn + next) - v;
      g.vs[s] = vs;
      g.adv[s] = adv;
      const float rc = fminf(fmaxf(ratio, lo), hi);
      const float a = ratio * adv, b = rc * adv;
      sum_pi -= fminf(a, b);
      const float dv = v - vs;
      sum_v += dv * dv;
      sum_ent -= ent;
      if (g.dvalues) g.dvalues[s] = 2.0f * g.critic_coef * dv * inv_m;
      if (g.dlogits) {
        const float dlp = a <= b ? -adv * ratio * inv_m : 0.0f;  // d L_pi / d logp_pi
        const float ce = g.entropy_coef * inv_m;
        const float* l = g.logits + s * g.sumA;
        float* d = g.dlogits + s * g.sumA;
        for (int k = 0; k < g.n_heads; ++k) {
          const int A = g.head_sizes[k];
          float mx = -INFINITY;
          for (int i = 0; i < A; ++i) mx = fmaxf(mx, l[i]);
          float se = 0.0f;
          for (int i = 0; i < A; ++i) se += expf(l[i] - mx);
          const float lse = mx + logf(se);
          float hk = 0.0f;
          for (int i = 0; i < A; ++i) {
            const float ls = l[i] - lse;
            hk -= expf(ls) * ls;
          }
          const int act = min(max(g.actions[s * g.n_heads + k], 0), A - 1);
          for (int i = 0; i < A; ++i) {
            const float ls = l[i] - lse;
            const float p = expf(ls);
            d[i] = dlp * ((i == act ? 1.0f : 0.0f) - p) + ce * p * (ls + hk);
          }
          l += A;
          d += A;
        }
      }
    }
  }
  sum_pi = wave_sum(sum_pi);
  sum_v = wave_sum(sum_v);
  sum_ent = wave_sum(sum_ent);
  if (lane == 0) {
    float* o = g.partials + (size_t)n * 4;
    o[0] = sum_pi;
    o[1] = sum_v;
    o[2] = sum_ent;
    o[3] = 0.0f;
  }
}

__global__ __launch_bounds__(kWave) void appo_reduce_kernel(const float* __restrict__ partials, int N,
                                                           float inv_m, float critic_coef,
                                                           float entropy_coef, float* __restrict__ loss) {
  const int lane = threadIdx.x;
  float a = 0.0f, b = 0.0f, c = 0.0f;
  for (int n = lane; n < N; n += kWave) {
    a += partials[(size_t)n * 4 + 0];
    b += partials[(size_t)n * 4 + 1];
    c += partials[(size_t)n * 4 + 2];
  }
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_sum(c);
  if (lane == 0) {
    const float l_pi = a * inv_m, l_v = critic_coef * b * inv_m, l_h = entropy_coef * c * inv_m;
    loss[0] = l_pi;
    loss[1] = l_v;
    loss[2] = l_h;
    loss[3] = l_pi + l_v + l_h;
  }
}

int check_loss_config(const sf_loss_config* c, const char* fn, int* sumA) {
  if (!c || c->struct_size != sizeof(sf_loss_config)) {
    set_error("%s: null configuration or struct_size mismatch", fn);
    return SF_ERR_ARG;
  }
  if (c->T < 1 || c->N < 1 || c->T > (1 << 20) || c->N > (1 << 24) || c->n_heads < 1 ||
      c->n_heads > SF_MAX_HEADS) {
    set_error("%s: T = %d, N = %d, n_heads = %d out of range", fn, c->T, c->N, c->n_heads);
    return SF_ERR_SHAPE;
  }
  int s = 0;
  for (int k = 0; k < c->n_heads; ++k) {
    if (c->head_sizes[k] < 1 || c->head_sizes[k] > 65535) {
      set_error("%s: head %d has size %d", fn, k, c->head_sizes[k]);
      return SF_ERR_SHAPE;
    }
    s += c->head_sizes[k];
  }
  if (!(c->clip >= 1.0f) || !(c->gamma >= 0.0f) || !(c->rho_bar > 0.0f) || !(c->c_bar > 0.0f)) {
    set_error("%s: clip must be >= 1, gamma >= 0, rho_bar and c_bar > 0", fn);
    return SF_ERR_SHAPE;
  }
  *sumA = s;
  return SF_OK;
}

}  // namespace
}  // namespace sf

using namespace sf;

extern "C" int64_t sf_appo_loss_workspace_bytes(const sf_loss_config* cfg) {
  int sumA;
  if (check_loss_config(cfg, "sf_appo_loss_workspace_bytes", &sumA) != SF_OK) return -1;
  return (int64_t)cfg->N * 4 * (int64_t)sizeof(float);
}

namespace {

// Argument checks and the two launches shared by the entry points; `partials` is device
// memory for N x 4 floats.
int run_appo_loss(const char* fn, const sf_loss_config* cfg, int sumA, const float* logits,
                  const int32_t* actions, const float* logp_mu, const float* values, const float* rewards,
                  const uint8_t* dones, float* vs, float* adv, float* loss, float* dlogits_opt,
                  float* dvalues_opt, float* partials, hipStream_t st) {
  if (!logits || !actions || !logp_mu || !values || !rewards || !dones || !vs || !adv || !loss ||
      !partials) {
    set_error("%s: null buffer", fn);
    return SF_ERR_ARG;
  }
  const void* al[] = {logits, actions, logp_mu, values, rewards, vs, adv, loss, dlogits_opt, dvalues_opt,
                      partials};
  for (const void* q : al)
    if ((reinterpret_cast<uintptr_t>(q) & 3) != 0) {
      set_error("%s: misaligned buffer (4 bytes)", fn);
      return SF_ERR_ARG;
    }
  LossArgs g;
  g.logits = logits; g.actions = actions; g.logp_mu = logp_mu; g.values = values; g.rewards = rewards;
  g.dones = dones; g.vs = vs; g.adv = adv; g.dlogits = dlogits_opt; g.dvalues = dvalues_opt;
  g.partials = partials;
  g.T = cfg->T; g.N = cfg->N; g.n_heads = cfg->n_heads; g.sumA = sumA;
  for (int k = 0; k < SF_MAX_HEADS; ++k) g.head_sizes[k] = k < cfg->n_heads ? cfg->head_sizes[k] : 0;
  g.gamma = cfg->gamma; g.rho_bar = cfg->rho_bar; g.c_bar = cfg->c_bar; g.clip = cfg->clip;
  g.critic_coef = cfg->critic_coef; g.entropy_coef = cfg->entropy_coef;
  const unsigned blocks = (unsigned)((cfg->N + kTrajPerBlock - 1) / kTrajPerBlock);
  appo_traj_kernel<<<blocks, kWave * kTrajPerBlock, 0, st>>>(g);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) {
    appo_reduce_kernel<<<1, kWave, 0, st>>>(g.partials, cfg->N, 1.0f / ((float)cfg->T * (float)cfg->N),
                                            cfg->critic_coef, cfg->entropy_coef, loss);
    e = hipGetLastError();
  }
  if (e != hipSuccess) {
    set_error("%s: launch failed: %s", fn, hipGetErrorString(e));
    return SF_ERR_DEVICE;
  }
  return SF_OK;
}

// Scratch of the entry point that allocates nothing: the per-trajectory partial sums.  One copy
// of this array exists on every GPU the library is loaded on, at an address of its own; host
// code never uses the symbol's name as an address but the pointer that hipGetSymbolAddress
// returns for the current device, looked up once per device.
constexpr int kStaticMaxTraj = 16384;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) float scratch[(size_t)kStaticMaxTraj * 4];
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(const char* fn, float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("%s: no current HIP device (%s)", fn, hipGetErrorString(e));
    return SF_ERR_DEVICE;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_error("%s: hipGetSymbolAddress failed on device %d: %s", fn, dev, hipGetErrorString(e));
      return SF_ERR_DEVICE;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SF_OK;
}

}  // namespace

extern "C" int sf_appo_loss(const sf_loss_config* cfg, const float* logits, const int32_t* actions,
                            const float* logp_mu, const float* values, const float* rewards,
                            const uint8_t* dones, float* vs, float* adv, float* loss,
                            float* dlogits_opt, float* dvalues_opt, void* workspace, void* hip_stream) {
  static const char* fn = "sf_appo_loss";
  int sumA;
  int rc = check_loss_config(cfg, fn, &sumA);
  if (rc != SF_OK) return rc;
  return run_appo_loss(fn, cfg, sumA, logits, actions, logp_mu, values, rewards, dones, vs, adv, loss,
                       dlogits_opt, dvalues_opt, (float*)workspace, reinterpret_cast<hipStream_t>(hip_stream));
}

extern "C" int32_t sf_appo_loss_static_max_trajectories(void) { return kStaticMaxTraj; }

extern "C" int sf_appo_loss_static(const sf_loss_config* cfg, const float* logits, const int32_t* actions,
                                   const float* logp_mu, const float* values, const float* rewards,
                                   const uint8_t* dones, float* vs, float* adv, float* loss,
                                   float* dlogits_opt, float* dvalues_opt, void* hip_stream) {
  static const char* fn = "sf_appo_loss_static";
  int sumA;
  int rc = check_loss_config(cfg, fn, &sumA);
  if (rc != SF_OK) return rc;
  if (cfg->N > kStaticMaxTraj) {
    set_error("%s: N = %d trajectories exceed the built-in scratch (%d); use sf_appo_loss with a workspace",
              fn, cfg->N, kStaticMaxTraj);
    return SF_ERR_SHAPE;
  }
  float* partials = nullptr;
  rc = static_scratch(fn, &partials);
  if (rc != SF_OK) return rc;
  // every trajectory's wave writes its slot before the reduction reads it: nothing to clear
  return run_appo_loss(fn, cfg, sumA, logits, actions, logp_mu, values, rewards, dones, vs, adv, loss,
                       dlogits_opt, dvalues_opt, partials, reinterpret_cast<hipStream_t>(hip_stream));
}

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
//
// Memory side: the arrays are time-major, so the 64 samples of a wave lie N * sumA floats apart
// and per-lane reads of a sample's logits touch a cache line per lane and element.  A workgroup
// therefore owns four consecutive trajectories: for every time step their logits (and actions)
// are one contiguous run in memory, which the 256 threads copy into LDS with coalesced loads
// (row pitch odd: the per-lane walks over a sample's logits are then free of bank conflicts);
// the lanes compute out of LDS, leave the logit gradients there in place, and the workgroup
// writes them back as contiguous runs.  Logits and actions cross the memory bus once.  Tiles
// that do not fit LDS (several hundred logits per sample) take the direct kernel.
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

// floor(e / d) for e < 2^20, 1 <= d < 2^12, through the multiplier m = ceil(2^32 / d) (exact in
// that range: the excess e * (m * d - 2^32) stays below 2^32); d = 1 has no 32-bit multiplier.
__host__ __device__ inline uint32_t magic_of(uint32_t d) {
  return d <= 1 ? 0u : (uint32_t)((0x100000000ull + d - 1) / d);
}
__device__ inline uint32_t div_magic(uint32_t e, uint32_t d, uint32_t m) { return d <= 1 ? e : __umulhi(e, m); }

struct LdsPlan {
  int pitch;             // floats per sample row of the logits tile (odd, >= sumA)
  uint32_t m_sumA, m_nh; // multipliers for division by sumA and by n_heads
  int vec4;              // logits rows may be copied as 16-byte pieces (pitch == sumA, alignment)
};

constexpr int kLossThreads = kWave * kTrajPerBlock;

// Tile copies between memory and LDS.  Row tt of the chunk holds, for time step t0 + tt, the nb
// trajectories' values side by side: memory run of nb * per elements at ((t0 + tt) * N + n0) * per,
// LDS sample (tt, j) at (tt * TPB + j) * pitch.  TO_LDS: memory -> LDS, else LDS -> memory.
// Loads are issued in batches of kCopyBatch per thread before the first of them is stored: a
// loop of load-then-store pays one memory latency per iteration.
constexpr int kCopyBatch = 8;

template <bool TO_LDS, int TPB, int NT, typename T>
__device__ inline void copy_tile(T* mem, T* tile, int t0, int nt, int N, int n0, int nb, int per,
                                 int pitch, uint32_t m_per) {
  const int rowlen = nb * per;
  const uint32_t m_row = magic_of((uint32_t)rowlen);
  const int total = nt * rowlen;
  for (int e0 = threadIdx.x; e0 < total; e0 += NT * kCopyBatch) {
    T v[kCopyBatch];
    T* dst[kCopyBatch];
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u) {
      const int e = e0 + u * NT;
      const int ec = e < total ? e : total - 1;
      const int tt = (int)div_magic((uint32_t)ec, (uint32_t)rowlen, m_row);
      const int r = ec - tt * rowlen;
      const int j = (int)div_magic((uint32_t)r, (uint32_t)per, m_per);
      const int i = r - j * per;
      T* gp = mem + ((size_t)(t0 + tt) * N + n0) * per + r;
      T* lp = tile + (tt * TPB + j) * pitch + i;
      v[u] = TO_LDS ? *gp : *lp;
      dst[u] = TO_LDS ? lp : gp;
    }
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u)
      if (e0 + u * NT < total) *dst[u] = v[u];
  }
}

// The same for a full-width tile (nb == TPB) whose rows are contiguous in LDS as in memory
// (pitch == per) and 16-byte aligned on both sides: 16-byte pieces.
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <bool TO_LDS, int TPB, int NT>
__device__ inline void copy_tile_vec4(float* mem, float* tile, int t0, int nt, int N, int n0, int per) {
  const int row4 = TPB * per / 4;  // pieces per row
  const uint32_t m_row = magic_of((uint32_t)row4);
  const int total = nt * row4;
  for (int e0 = threadIdx.x; e0 < total; e0 += NT * kCopyBatch) {
    f32x4 v[kCopyBatch];
    f32x4* dst[kCopyBatch];
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u) {
      const int e = e0 + u * NT;
      const int ec = e < total ? e : total - 1;
      const int tt = (int)div_magic((uint32_t)ec, (uint32_t)row4, m_row);
      const int r = ec - tt * row4;
      f32x4* gp = (f32x4*)(mem + ((size_t)(t0 + tt) * N + n0) * per) + r;
      f32x4* lp = (f32x4*)(tile + (size_t)tt * TPB * per) + r;
      v[u] = TO_LDS ? *gp : *lp;
      dst[u] = TO_LDS ? lp : gp;
    }
#pragma unroll
    for (int u = 0; u < kCopyBatch; ++u)
      if (e0 + u * NT < total) *dst[u] = v[u];
  }
}

// LW lanes per trajectory: 64, or 32 when T <= 32 (two trajectories per wave, no idle half);
// NT threads per workgroup (LW = 32: two waves, so that the grid has several workgroups per CU
// and one's tile copies overlap another's arithmetic).
// Per head the forward pass takes one exponential per logit:
//   d_i = l_i - max, e_i = exp(d_i), se = sum e_i, sd = sum e_i d_i
//   lse = max + log se,  entropy = log se - sd / se   (= -sum p_i (l_i - lse))
// (lse, entropy) of every head of every sample are kept in LDS for the gradient pass, which takes
// one more exponential per logit (p_i = exp(l_i - lse)).  These exponentials (arguments <= 0,
// results only ever summed or multiplied into terms of the 1e-4 tolerance) use the hardware
// exp2 (about 2 ulp for arguments of a few units); the logarithm per head and the importance
// ratio stay on the accurate routines.
template <int LW, int NT>
__global__ __launch_bounds__(NT) void appo_traj_lds_kernel(LossArgs g, LdsPlan plan) {
  constexpr int TPB = NT / LW;  // trajectories per workgroup
  extern __shared__ __attribute__((aligned(16))) float lds_tile[];
  float* ltile = lds_tile;                                   // [LW][TPB][pitch] logits, then gradients
  float* htile = ltile + LW * TPB * plan.pitch;              // [LW][TPB][n_heads][2] (lse, entropy)
  int32_t* atile = (int32_t*)(htile + LW * TPB * g.n_heads * 2);  // [LW][TPB][n_heads]
  const int lane = threadIdx.x % LW, j = threadIdx.x / LW;
  const int n0 = blockIdx.x * TPB;
  const int nb = g.N - n0 < TPB ? g.N - n0 : TPB;
  const int n = n0 + j;
  const bool have = n < g.N;  // lanes without a trajectory only help with the copies
  const bool vec4 = plan.vec4 && nb == TPB;
  const float inv_m = 1.0f / ((float)g.T * (float)g.N);
  const float lo = 1.0f / g.clip, hi = g.clip;
  float sum_pi = 0.0f, sum_v = 0.0f, sum_ent = 0.0f;
  float carry = 0.0f;
  const int n_chunks = (g.T + LW - 1) / LW;
  for (int ch = n_chunks - 1; ch >= 0; --ch) {
    const int t0 = ch * LW;
    const int nt = g.T - t0 < LW ? g.T - t0 : LW;
    // the sample's scalars are requested first: their latency passes under the tile copies
    const int tt = t0 + lane < g.T ? lane : nt - 1;  // idle lanes re-read the chunk's last step
    const size_t s = (size_t)(t0 + tt) * g.N + (have ? n : g.N - 1);
    const float v = g.values[s], vn = g.values[s + g.N], r = g.rewards[s], lmu = g.logp_mu[s];
    const float gm = g.dones[s] ? 0.0f : g.gamma;
    if (vec4)
      copy_tile_vec4<true, TPB, NT>(const_cast<float*>(g.logits), ltile, t0, nt, g.N, n0, g.sumA);
    else
      copy_tile<true, TPB, NT>(const_cast<float*>(g.logits), ltile, t0, nt, g.N, n0, nb, g.sumA, plan.pitch,
                           plan.m_sumA);
    copy_tile<true, TPB, NT>(const_cast<int32_t*>(g.actions), atile, t0, nt, g.N, n0, nb, g.n_heads, g.n_heads,
                         plan.m_nh);
    __syncthreads();
    if (have) {
      const bool live = t0 + lane < g.T;
      const int smp = tt * TPB + j;
      float* l0 = ltile + smp * plan.pitch;
      float* h0 = htile + smp * g.n_heads * 2;
      const int32_t* a0 = atile + smp * g.n_heads;
      float logp = 0.0f, ent = 0.0f;
      {
        const float* l = l0;
        for (int k = 0; k < g.n_heads; ++k) {
          const int A = g.head_sizes[k];
          // four independent chains per pass: with one wave per SIMD there is nobody else to
          // hide the latency of an LDS read or of an exponential behind
          float m4[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
          int i = 0;
          for (; i + 4 <= A; i += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) m4[u] = fmaxf(m4[u], l[i + u]);
          }
          for (; i < A; ++i) m4[0] = fmaxf(m4[0], l[i]);
          const float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
          float se4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, sd4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          for (i = 0; i + 4 <= A; i += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const float d = l[i + u] - mx;
              const float e = __expf(d);
              se4[u] += e;
              sd4[u] = fmaf(e, d, sd4[u]);
            }
          }
          for (; i < A; ++i) {
            const float d = l[i] - mx;
            const float e = __expf(d);
            se4[0] += e;
            sd4[0] = fmaf(e, d, sd4[0]);
          }
          const float se = (se4[0] + se4[1]) + (se4[2] + se4[3]);
          const float sd = (sd4[0] + sd4[1]) + (sd4[2] + sd4[3]);
          const float lg = logf(se);
          const float lse = mx + lg, hk = lg - sd / se;
          if (live) {  // (idle lanes share the last step's slot with its owner)
            h0[2 * k] = lse;
            h0[2 * k + 1] = hk;
          }
          const int a = min(max(a0[k], 0), A - 1);
          logp += l[a] - lse;
          ent += hk;
          l += A;
        }
      }
      const float ratio = expf(logp - lmu);
      const float rho = fminf(g.rho_bar, ratio), c = fminf(g.c_bar, ratio);
      const float delta = live ? rho * (r + gm * vn - v) : 0.0f;
      const float gc = live ? gm * c : 0.0f;
      float x = carry, mine = 0.0f;
      for (int l = LW - 1; l >= 0; --l) {
        x = __shfl(delta, l, LW) + __shfl(gc, l, LW) * x;
        if (lane == l) mine = x;
      }
      float next = __shfl_down(mine, 1, LW);
      if (lane == LW - 1) next = carry;
      carry = __shfl(mine, 0, LW);
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
          float* l = l0;  // the gradient replaces the logits in the tile
          for (int k = 0; k < g.n_heads; ++k) {
            const int A = g.head_sizes[k];
            const float lse = h0[2 * k], hk = h0[2 * k + 1];
            const int act = min(max(a0[k], 0), A - 1);
            int i = 0;
            for (; i + 4 <= A; i += 4) {
              float q[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) q[u] = l[i + u];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const float ls = q[u] - lse;
                const float p = __expf(ls);
                q[u] = dlp * ((i + u == act ? 1.0f : 0.0f) - p) + ce * p * (ls + hk);
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) l[i + u] = q[u];
            }
            for (; i < A; ++i) {
              const float ls = l[i] - lse;
              const float p = __expf(ls);
              l[i] = dlp * ((i == act ? 1.0f : 0.0f) - p) + ce * p * (ls + hk);
            }
            l += A;
          }
        }
      }
    }
    __syncthreads();
    if (g.dlogits) {
      if (vec4)
        copy_tile_vec4<false, TPB, NT>(g.dlogits, ltile, t0, nt, g.N, n0, g.sumA);
      else
        copy_tile<false, TPB, NT>(g.dlogits, ltile, t0, nt, g.N, n0, nb, g.sumA, plan.pitch, plan.m_sumA);
    }
    __syncthreads();  // the tiles are free for the next chunk
  }
  if (have) {
#pragma unroll
    for (int m = LW / 2; m >= 1; m >>= 1) {
      sum_pi += __shfl_xor(sum_pi, m, LW);
      sum_v += __shfl_xor(sum_v, m, LW);
      sum_ent += __shfl_xor(sum_ent, m, LW);
    }
    if (lane == 0) {
      float* o = g.partials + (size_t)n * 4;
      o[0] = sum_pi;
      o[1] = sum_v;
      o[2] = sum_ent;
      o[3] = 0.0f;
    }
  }
}

// Adds the per-trajectory partial sums in an order that depends on N only: thread i takes
// entries i, i + 256, ... (independent 16-byte loads), then a fixed binary tree over the 256
// threads' sums in LDS.
constexpr int kReduceThreads = 256;
__global__ __launch_bounds__(kReduceThreads) void appo_reduce_kernel(const float* __restrict__ partials, int N,
                                                                     float inv_m, float critic_coef,
                                                                     float entropy_coef, float* __restrict__ loss) {
  __shared__ float red[3][kReduceThreads];
  const int tid = threadIdx.x;
  float a = 0.0f, b = 0.0f, c = 0.0f;
  for (int n = tid; n < N; n += kReduceThreads) {
    const f32x4 p = *(const f32x4*)(partials + (size_t)n * 4);
    a += p[0];
    b += p[1];
    c += p[2];
  }
  red[0][tid] = a;
  red[1][tid] = b;
  red[2][tid] = c;
  __syncthreads();
  for (int m = kReduceThreads / 2; m >= 1; m >>= 1) {
    if (tid < m) {
      red[0][tid] += red[0][tid + m];
      red[1][tid] += red[1][tid + m];
      red[2][tid] += red[2][tid + m];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const float l_pi = red[0][0] * inv_m, l_v = critic_coef * red[1][0] * inv_m,
                l_h = entropy_coef * red[2][0] * inv_m;
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
  // N x 4 partial sums, plus room to move a 4-byte aligned pointer up to a 16-byte boundary
  return (int64_t)cfg->N * 4 * (int64_t)sizeof(float) + 16;
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
  // the LDS-staged kernel where a chunk's tiles fit LDS, with 32 lanes per trajectory (eight
  // trajectories per workgroup) when the trajectories are no longer than that
  const int LW = cfg->T <= 32 ? 32 : 64;
  const int NT = LW == 32 ? 128 : 256;
  const int TPB = NT / LW;
  LdsPlan plan;
  plan.pitch = sumA | 1;
  plan.m_sumA = magic_of((uint32_t)sumA);
  plan.m_nh = magic_of((uint32_t)cfg->n_heads);
  plan.vec4 = plan.pitch == sumA && (TPB * sumA) % 4 == 0 && ((size_t)cfg->N * sumA) % 4 == 0 &&
              ((uintptr_t)logits & 15) == 0 && (!dlogits_opt || ((uintptr_t)dlogits_opt & 15) == 0);
  const size_t lds = sizeof(float) * NT * ((size_t)plan.pitch + 3 * (size_t)cfg->n_heads);
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&] {
    attr_status = hipFuncSetAttribute((const void*)appo_traj_lds_kernel<32, 128>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (attr_status == hipSuccess)
      attr_status = hipFuncSetAttribute((const void*)appo_traj_lds_kernel<64, 256>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
  });
  if (attr_status != hipSuccess) {
    set_error("%s: hipFuncSetAttribute failed: %s", fn, hipGetErrorString(attr_status));
    return SF_ERR_DEVICE;
  }
  const unsigned blocks = (unsigned)((cfg->N + TPB - 1) / TPB);
  if (lds <= 128 * 1024) {
    if (LW == 32)
      appo_traj_lds_kernel<32, 128><<<blocks, 128, lds, st>>>(g, plan);
    else
      appo_traj_lds_kernel<64, 256><<<blocks, 256, lds, st>>>(g, plan);
  } else {
    appo_traj_kernel<<<(unsigned)((cfg->N + kTrajPerBlock - 1) / kTrajPerBlock), kLossThreads, 0, st>>>(g);
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) {
    appo_reduce_kernel<<<1, kReduceThreads, 0, st>>>(g.partials, cfg->N, 1.0f / ((float)cfg->T * (float)cfg->N),
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
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 3) != 0) {
    set_error("%s: null or misaligned workspace", fn);
    return SF_ERR_ARG;
  }
  return run_appo_loss(fn, cfg, sumA, logits, actions, logp_mu, values, rewards, dones, vs, adv, loss,
                       dlogits_opt, dvalues_opt,
                       reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(workspace) + 15) & ~(uintptr_t)15),
                       reinterpret_cast<hipStream_t>(hip_stream));
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

// Action heads, value head, log-probability and sampling: one 64-lane wavefront
// per batch row.
//
// The linear heads (paper, App. "Model architectures": a pair of fully connected
// layers giving the action distribution and the baseline) are thin dot products
// over h_out.  Each categorical head is then sampled with the Gumbel-max rule:
// category i is perturbed with g_i = -log(-log(u_i)), u_i from a counter-based
// Philox4x32-10 stream keyed by (seed; row, step, head, i/4), and the lowest index
// attaining the maximum is the action.  Heads are independent (paper, App.
// "VizDoom experiments"), so the joint log-probability is the sum over heads.
#include "sf_internal.h"

namespace sf {

namespace {

constexpr int kWave = 64;
constexpr int kRowsPerBlock = 4;
constexpr int kMaxLogits = 1024;  // per row, value included (LDS staging)

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                     uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t m0 = 0xD2511F53u, m1 = 0xCD9E8D57u;
    uint32_t hi0 = __umulhi(m0, c0), lo0 = m0 * c0;
    uint32_t hi1 = __umulhi(m1, c2), lo1 = m1 * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}

__global__ __launch_bounds__(kWave* kRowsPerBlock) void heads_kernel(
    const float* __restrict__ h, const float* __restrict__ head_w,
    const float* __restrict__ head_b, const int32_t* __restrict__ head_off, int B, int H,
    int n_heads, int sumA, uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo,
    uint32_t step_hi, int32_t* __restrict__ actions, float* __restrict__ logp,
    float* __restrict__ value, float* __restrict__ logits_opt, const int32_t* __restrict__ ids,
    float* __restrict__ h_table, int n_env, int S, int lane_per_head) {
  __shared__ float s_logits[kRowsPerBlock][kMaxLogits];
  __shared__ float s_pert[kRowsPerBlock][kMaxLogits];
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int b = blockIdx.x * kRowsPerBlock + wave;
  if (b >= B) return;  // whole wave leaves together; no block-level barrier below
  float* lg = s_logits[wave];
  float* pt = s_pert[wave];
  // state rows hold S >= H floats; the heads read the first H (an LSTM's h)
  const float* hp = h + (size_t)b * S;
  // With ids, the row stands for environment ids[b]: that is the sampler's counter word, and
  // the row's new state goes back to row ids[b] of the state table (ids outside the table
  // write nothing).
  const uint32_t env = ids ? (uint32_t)ids[b] : (uint32_t)b;
  if (h_table && env < (uint32_t)n_env)
    for (int i = lane; i < S; i += kWave) h_table[(size_t)env * S + i] = hp[i];

  // Logits and value: lane-strided dot products, eight outputs at a time so that their
  // loads are all in flight together.  The eight partial sums per lane are reduced over
  // the wave by a transposing butterfly (fixed order): at distance 32, 16 and 8 each lane
  // hands half of its remaining outputs to its partner and adds the partner's share of the
  // other half, so an 8-lane group ends up with one output, which three more steps finish:
  // 10 cross-lane moves for 8 outputs instead of 48.
  constexpr int kGroup = 8;
  const bool b5 = (lane & 32) != 0, b4 = (lane & 16) != 0, b3 = (lane & 8) != 0;
  const int u_own = (b5 ? 4 : 0) + (b4 ? 2 : 0) + (b3 ? 1 : 0);
  for (int a0 = 0; a0 <= sumA; a0 += kGroup) {
    float part[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u) part[u] = 0.0f;
    const float* wrow[kGroup];
#pragma unroll
    for (int u = 0; u < kGroup; ++u)  // clamp: duplicates are computed but not stored
      wrow[u] = head_w + (size_t)(a0 + u <= sumA ? a0 + u : sumA) * H;
#pragma unroll 4
    for (int i = lane; i < H; i += kWave) {
      const float hv = hp[i];
#pragma unroll
      for (int u = 0; u < kGroup; ++u) part[u] = fmaf(hv, wrow[u][i], part[u]);
    }
    float q4[4], q2[2];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      q4[u] = (b5 ? part[u + 4] : part[u]) + __shfl_xor(b5 ? part[u] : part[u + 4], 32, kWave);
#pragma unroll
    for (int u = 0; u < 2; ++u)
      q2[u] = (b4 ? q4[u + 2] : q4[u]) + __shfl_xor(b4 ? q4[u] : q4[u + 2], 16, kWave);
    float q1 = (b3 ? q2[1] : q2[0]) + __shfl_xor(b3 ? q2[0] : q2[1], 8, kWave);
    q1 += __shfl_xor(q1, 4, kWave);
    q1 += __shfl_xor(q1, 2, kWave);
    q1 += __shfl_xor(q1, 1, kWave);
    const int a = a0 + u_own;
    if (a <= sumA && (lane & 7) == 0) lg[a] = q1 + head_b[a];
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();
  if (lane == 0) value[b] = lg[sumA];
  if (logits_opt)
    for (int a = lane; a < sumA; a += kWave) logits_opt[(size_t)b * sumA + a] = lg[a];
  if (!actions) return;  // (the learner's pass wants logits and value only)

  // Gumbel perturbation of every logit of every head in one pass over the lanes.
  for (int idx = lane; idx < sumA; idx += kWave) {
    int k = 0;
    while (head_off[k + 1] <= idx) ++k;
    const int i = idx - head_off[k];
    uint32_t wd[4];
    philox4x32_10(env, step_lo, step_hi, ((uint32_t)k << 16) | (uint32_t)(i >> 2), seed_lo, seed_hi,
                  wd);
    const uint32_t word = wd[i & 3];
    const float u = ((float)(word >> 9) + 0.5f) * 0x1.0p-23f;
    pt[idx] = lg[idx] + -logf(-logf(u));
  }
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();

  float lp_total = 0.0f;
  if (lane_per_head) {
    // Several small heads (none above 32 categories): lane k finishes head k on its own, all
    // heads side by side, instead of one wave-wide butterfly per head after another.  Categories
    // are visited in ascending order, so the first maximum wins ties.
    float lp = 0.0f;
    if (lane < n_heads) {
      const int off = head_off[lane];
      const int A = head_off[lane + 1] - off;
      float best = pt[off], lmax = lg[off];
      int arg = 0;
      for (int i = 1; i < A; ++i) {
        const float pert = pt[off + i];
        if (pert > best) {
          best = pert;
          arg = i;
        }
        lmax = fmaxf(lmax, lg[off + i]);
      }
      float se = 0.0f;
      for (int i = 0; i < A; ++i) se += expf(lg[off + i] - lmax);
      lp = lg[off + arg] - (lmax + logf(se));
      actions[(size_t)b * n_heads + lane] = arg;
    }
    lp_total = wave_sum(lp);
  } else
  for (int k = 0; k < n_heads; ++k) {
    const int off = head_off[k];
    const int A = head_off[k + 1] - off;
    float best = -INFINITY, lmax = -INFINITY;
    int arg = 0x7FFFFFFF;
    for (int i = lane; i < A; i += kWave) {
      const float pert = pt[off + i];
      if (arg == 0x7FFFFFFF || pert > best) {
        best = pert;
        arg = i;
      }
      lmax = fmaxf(lmax, lg[off + i]);
    }
    // Butterfly over the lanes that hold categories: P = the power of two covering
    // min(A, 64); lanes below P end with the result, lane 0 broadcasts it.
    int P = 1;
    while (P < A && P < kWave) P <<= 1;
    // argmax, ties to the lowest index
    for (int m = P >> 1; m >= 1; m >>= 1) {
      const float ob = __shfl_xor(best, m, kWave);
      const int oa = __shfl_xor(arg, m, kWave);
      const bool take = (oa != 0x7FFFFFFF) && (arg == 0x7FFFFFFF || ob > best || (ob == best && oa < arg));
      if (take) {
        best = ob;
        arg = oa;
      }
      lmax = fmaxf(lmax, __shfl_xor(lmax, m, kWave));
    }
    arg = __shfl(arg, 0, kWave);
    lmax = __shfl(lmax, 0, kWave);
    float se = 0.0f;
    for (int i = lane; i < A; i += kWave) se += expf(lg[off + i] - lmax);
    for (int m = P >> 1; m >= 1; m >>= 1) se += __shfl_xor(se, m, kWave);
    se = __shfl(se, 0, kWave);
    const float lse = lmax + logf(se);
    lp_total += lg[off + arg] - lse;
    if (lane == 0) actions[(size_t)b * n_heads + k] = arg;
  }
  if (lane == 0) logp[b] = lp_total;
}

}  // namespace

hipError_t launch_heads(int B, int H, int n_heads, int sumA, const int32_t* head_off,
                        const float* h, const float* head_w, const float* head_b, uint64_t seed,
                        uint64_t step, int32_t* actions, float* logp, float* value,
                        float* logits_opt, const int32_t* ids, float* h_table, int n_env,
                        int state_dim, int max_head, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (sumA + 1 > kMaxLogits) return hipErrorInvalidValue;
  unsigned blocks = (unsigned)((B + kRowsPerBlock - 1) / kRowsPerBlock);
  heads_kernel<<<blocks, kWave * kRowsPerBlock, 0, st>>>(
      h, head_w, head_b, head_off, B, H, n_heads, sumA, (uint32_t)seed, (uint32_t)(seed >> 32),
      (uint32_t)step, (uint32_t)(step >> 32), actions, logp, value, logits_opt, ids, h_table,
      n_env, state_dim, (n_heads > 1 && n_heads <= kWave && max_head <= 32) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace sf

// Shape-agnostic kernels: one thread per output element, fp32 FMA in a fixed
// order.  They serve every network description the boundary accepts; the
// MFMA kernels replace them for the shapes they are specialised for.
#include "sf_internal.h"

namespace sf {

namespace {

constexpr int kThreads = 256;

// Convolution (paper, App. "Model architectures": convolutional encoder).
// in: planar bytes [B][C][H][W] (normalised on the fly) or channels-last fp32.
// out: channels-last fp32 [B][Ho][Wo][Cout].  w: [k][k][Cin][Cout].
template <bool kU8Planar>
__global__ __launch_bounds__(kThreads) void conv_generic_kernel(
    const void* __restrict__ in_v, float* __restrict__ out, const float* __restrict__ w,
    const float* __restrict__ bias, const float* __restrict__ residual, long long total, int Cin,
    int H, int W, int Cout, int k, int s, int pad, int Ho, int Wo, int relu_in, int relu_out,
    float obs_sub, float obs_mul) {
  long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  int o = (int)(idx % Cout);
  long long t = idx / Cout;
  int ox = (int)(t % Wo);
  t /= Wo;
  int oy = (int)(t % Ho);
  long long b = t / Ho;
  float acc = bias[o];
  for (int p = 0; p < k; ++p) {
    int y = oy * s + p - pad;
    if (y < 0 || y >= H) continue;
    for (int q = 0; q < k; ++q) {
      int x = ox * s + q - pad;
      if (x < 0 || x >= W) continue;
      const float* wp = w + ((size_t)(p * k + q) * Cin) * Cout + o;
      if (kU8Planar) {
        const uint8_t* ip = (const uint8_t*)in_v + ((size_t)b * Cin * H + y) * W + x;
        for (int c = 0; c < Cin; ++c) {
          float v = ((float)ip[(size_t)c * H * W] - obs_sub) * obs_mul;
          acc = fmaf(v, wp[(size_t)c * Cout], acc);
        }
      } else {
        const float* ip = (const float*)in_v + (((size_t)b * H + y) * W + x) * Cin;
        for (int c = 0; c < Cin; ++c) {
          float v = ip[c];
          if (relu_in) v = fmaxf(v, 0.0f);
          acc = fmaf(v, wp[(size_t)c * Cout], acc);
        }
      }
    }
  }
  if (residual) acc += residual[idx];
  if (relu_out) acc = fmaxf(acc, 0.0f);
  out[idx] = acc;
}

// 3x3/s2 max pooling whose padding ring never wins (channels-last).
__global__ __launch_bounds__(kThreads) void maxpool_kernel(const float* __restrict__ in,
                                                           float* __restrict__ out,
                                                           long long total, int C, int H, int W,
                                                           int Ho, int Wo) {
  long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  int c = (int)(idx % C);
  long long t = idx / C;
  int ox = (int)(t % Wo);
  t /= Wo;
  int oy = (int)(t % Ho);
  long long b = t / Ho;
  float m = -INFINITY;
  for (int y = 2 * oy - 1; y <= 2 * oy + 1; ++y) {
    if (y < 0 || y >= H) continue;
    for (int x = 2 * ox - 1; x <= 2 * ox + 1; ++x) {
      if (x < 0 || x >= W) continue;
      m = fmaxf(m, in[(((size_t)b * H + y) * W + x) * C + c]);
    }
  }
  out[idx] = m;
}

// out[b][o] = act(bias[o] + sum_i in[b][i] * w_t[i][o])
__global__ __launch_bounds__(kThreads) void linear_generic_kernel(
    const float* __restrict__ in, const float* __restrict__ w_t, const float* __restrict__ bias,
    float* __restrict__ out, int n_in, int n_out, int relu) {
  int o = blockIdx.x * kThreads + threadIdx.x;
  int b = blockIdx.y;
  if (o >= n_out) return;
  const float* ip = in + (size_t)b * n_in;
  float acc = bias[o];
  for (int i = 0; i < n_in; ++i) acc = fmaf(ip[i], w_t[(size_t)i * n_out + o], acc);
  if (relu) acc = fmaxf(acc, 0.0f);
  out[(size_t)b * n_out + o] = acc;
}

// Measurement encoder of the full architecture: one or two fully connected + ReLU layers
// in one launch.  A workgroup handles kMeasRows rows; the rows' inputs and the hidden
// activations sit in LDS, every weight is read once per workgroup.  Sums run in the same
// order as linear_generic_kernel's.
constexpr int kMeasRows = 4;
constexpr int kMeasThreads = 128;

__global__ __launch_bounds__(kMeasThreads) void meas_mlp_kernel(
    const float* __restrict__ meas, int B, int n0, const float* __restrict__ w1_t,
    const float* __restrict__ b1, int n1, const float* __restrict__ w2_t,
    const float* __restrict__ b2, int n2, float* __restrict__ out) {
  extern __shared__ float sm[];
  float* s_in = sm;                   // [kMeasRows][n0]
  float* s_h = sm + kMeasRows * n0;   // [kMeasRows][n1]
  const int r0 = blockIdx.x * kMeasRows;
  const int tid = threadIdx.x;
  for (int i = tid; i < kMeasRows * n0; i += kMeasThreads) {
    const int r = i / n0;
    s_in[i] = r0 + r < B ? meas[(size_t)(r0 + r) * n0 + (i - r * n0)] : 0.0f;
  }
  __syncthreads();
  for (int o = tid; o < n1; o += kMeasThreads) {
    float acc[kMeasRows];
#pragma unroll
    for (int r = 0; r < kMeasRows; ++r) acc[r] = b1[o];
#pragma unroll 8
    for (int i = 0; i < n0; ++i) {
      const float w = w1_t[(size_t)i * n1 + o];
#pragma unroll
      for (int r = 0; r < kMeasRows; ++r) acc[r] = fmaf(s_in[r * n0 + i], w, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < kMeasRows; ++r) {
      const float v = fmaxf(acc[r], 0.0f);
      if (n2 > 0)
        s_h[r * n1 + o] = v;
      else if (r0 + r < B)
        out[(size_t)(r0 + r) * n1 + o] = v;
    }
  }
  if (n2 == 0) return;
  __syncthreads();
  for (int o = tid; o < n2; o += kMeasThreads) {
    float acc[kMeasRows];
#pragma unroll
    for (int r = 0; r < kMeasRows; ++r) acc[r] = b2[o];
#pragma unroll 8
    for (int i = 0; i < n1; ++i) {
      const float w = w2_t[(size_t)i * n2 + o];
#pragma unroll
      for (int r = 0; r < kMeasRows; ++r) acc[r] = fmaf(s_h[r * n1 + i], w, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < kMeasRows; ++r)
      if (r0 + r < B) out[(size_t)(r0 + r) * n2 + o] = fmaxf(acc[r], 0.0f);
  }
}

__device__ inline float sigmoidf_acc(float a) { return 1.0f / (1.0f + expf(-a)); }

// Recurrent cell (GRU or LSTM) with the episode-boundary reset applied to the incoming
// state, any sizes.  One thread per (row, hidden unit).  The input features come in one or
// two pieces (x2 may be null); the transposed weights have one column block of H per gate:
// GRU r, z, n; LSTM i, f, g, o.  State rows hold H floats (GRU) or [h | c] (LSTM).
template <bool LSTM>
__global__ __launch_bounds__(kThreads) void rnn_generic_kernel(
    const float* __restrict__ x1, int n1, const float* __restrict__ x2, int n2,
    const float* __restrict__ h_in, const uint8_t* __restrict__ done,
    const float* __restrict__ wih_t, const float* __restrict__ whh_t,
    const float* __restrict__ bih, const float* __restrict__ bhh, float* __restrict__ h_out,
    int H, const int32_t* __restrict__ ids, int n_env) {
  constexpr int G = LSTM ? 4 : 3;
  const int S = LSTM ? 2 * H : H;
  int j = blockIdx.x * kThreads + threadIdx.x;
  int b = blockIdx.y;
  if (j >= H) return;
  bool reset = done[b] != 0;
  // with ids, the row's state is row ids[b] of a table; an id outside it reads as zero state
  int hb = b;
  if (ids) {
    const int e = ids[b];
    const bool ok = (unsigned)e < (unsigned)n_env;
    hb = ok ? e : 0;
    reset = reset || !ok;
  }
  const float* hp = h_in + (size_t)hb * S;
  float gi[G], gh[G];
#pragma unroll
  for (int q = 0; q < G; ++q) {
    gi[q] = bih[q * H + j];
    gh[q] = bhh[q * H + j];
  }
  for (int i = 0; i < n1 + n2; ++i) {
    const float v = i < n1 ? x1[(size_t)b * n1 + i] : x2[(size_t)b * n2 + (i - n1)];
    const float* wp = wih_t + (size_t)i * G * H + j;
#pragma unroll
    for (int q = 0; q < G; ++q) gi[q] = fmaf(v, wp[q * H], gi[q]);
  }
  if (!reset) {
    for (int i = 0; i < H; ++i) {
      const float v = hp[i];
      const float* wp = whh_t + (size_t)i * G * H + j;
#pragma unroll
      for (int q = 0; q < G; ++q) gh[q] = fmaf(v, wp[q * H], gh[q]);
    }
  }
  if (LSTM) {
    const float cprev = reset ? 0.0f : hp[H + j];
    const float ig = sigmoidf_acc(gi[0] + gh[0]);
    const float fg = sigmoidf_acc(gi[1] + gh[1]);
    const float gg = tanhf(gi[2] + gh[2]);
    const float og = sigmoidf_acc(gi[G - 1] + gh[G - 1]);
    const float cn = fg * cprev + ig * gg;
    h_out[(size_t)b * S + H + j] = cn;
    h_out[(size_t)b * S + j] = og * tanhf(cn);
  } else {
    const float hprev = reset ? 0.0f : hp[j];
    const float r = sigmoidf_acc(gi[0] + gh[0]);
    const float z = sigmoidf_acc(gi[1] + gh[1]);
    const float n = tanhf(gi[2] + r * gh[2]);
    h_out[(size_t)b * S + j] = (1.0f - z) * n + z * hprev;
  }
}


// Plain copy of 16-byte words: the known-size reference for scaling HBM byte counters.
__global__ __launch_bounds__(kThreads) void copy16_kernel(const uint4* __restrict__ src,
                                                          uint4* __restrict__ dst, long long n16) {
  long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long stride = (long long)gridDim.x * kThreads;
  for (; i < n16; i += stride) dst[i] = src[i];
}

inline unsigned blocks_for(long long total) { return (unsigned)((total + kThreads - 1) / kThreads); }

}  // namespace

hipError_t launch_conv_generic(const ConvLayer& L, int B, const void* in, bool in_is_u8_planar,
                               float obs_sub, float obs_mul, const float* residual, float* out,
                               hipStream_t st) {
  long long total = (long long)B * L.Ho * L.Wo * L.cout;
  if (total == 0) return hipSuccess;
  if (in_is_u8_planar)
    conv_generic_kernel<true><<<blocks_for(total), kThreads, 0, st>>>(
        in, out, L.w_khwc_o, L.bias, residual, total, L.cin, L.H, L.W, L.cout, L.k, L.s, L.pad,
        L.Ho, L.Wo, L.relu_in, L.relu_out, obs_sub, obs_mul);
  else
    conv_generic_kernel<false><<<blocks_for(total), kThreads, 0, st>>>(
        in, out, L.w_khwc_o, L.bias, residual, total, L.cin, L.H, L.W, L.cout, L.k, L.s, L.pad,
        L.Ho, L.Wo, L.relu_in, L.relu_out, obs_sub, obs_mul);
  return hipGetLastError();
}

hipError_t launch_maxpool3x3s2p1(int B, int C, int H, int W, const float* in, float* out,
                                 hipStream_t st) {
  int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  long long total = (long long)B * Ho * Wo * C;
  if (total == 0) return hipSuccess;
  maxpool_kernel<<<blocks_for(total), kThreads, 0, st>>>(in, out, total, C, H, W, Ho, Wo);
  return hipGetLastError();
}

hipError_t launch_linear_generic(int B, int n_in, int n_out, const float* in, const float* w_t,
                                 const float* bias, int relu, float* out, hipStream_t st) {
  if (B == 0) return hipSuccess;
  dim3 grid((n_out + kThreads - 1) / kThreads, B);
  linear_generic_kernel<<<grid, kThreads, 0, st>>>(in, w_t, bias, out, n_in, n_out, relu);
  return hipGetLastError();
}

bool meas_mlp_supported(int n0, int n1) { return (size_t)kMeasRows * (n0 + n1) * sizeof(float) <= 48 * 1024; }

// w1_t [n0][n1], w2_t [n1][n2] (transposed weights); n2 == 0: a single layer.
// out [B][n2 ? n2 : n1].
hipError_t launch_meas_mlp(int B, int n0, const float* meas, const float* w1_t, const float* b1, int n1,
                           const float* w2_t, const float* b2, int n2, float* out, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (!meas_mlp_supported(n0, n1)) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((B + kMeasRows - 1) / kMeasRows);
  const size_t lds = (size_t)kMeasRows * (n0 + n1) * sizeof(float);
  meas_mlp_kernel<<<blocks, kMeasThreads, lds, st>>>(meas, B, n0, w1_t, b1, n1, w2_t, b2, n2, out);
  return hipGetLastError();
}

hipError_t launch_rnn_generic(int lstm, int B, int n1, int n2, int H, const float* x1, const float* x2,
                              const float* h_in, const uint8_t* done, const float* wih_t,
                              const float* whh_t, const float* bih, const float* bhh, float* h_out,
                              const int32_t* ids, int n_env, hipStream_t st) {
  if (B == 0) return hipSuccess;
  dim3 grid((H + kThreads - 1) / kThreads, B);
  if (!x2) n2 = 0;
  if (lstm)
    rnn_generic_kernel<true><<<grid, kThreads, 0, st>>>(x1, n1, x2, n2, h_in, done, wih_t, whh_t, bih,
                                                        bhh, h_out, H, ids, n_env);
  else
    rnn_generic_kernel<false><<<grid, kThreads, 0, st>>>(x1, n1, x2, n2, h_in, done, wih_t, whh_t, bih,
                                                         bhh, h_out, H, ids, n_env);
  return hipGetLastError();
}

hipError_t launch_copy16(const void* src, void* dst, long long bytes, hipStream_t st) {
  long long n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  long long blocks = (n16 + kThreads - 1) / kThreads;
  if (blocks > 256 * 32) blocks = 256 * 32;
  copy16_kernel<<<(unsigned)blocks, kThreads, 0, st>>>((const uint4*)src, (uint4*)dst, n16);
  return hipGetLastError();
}

}  // namespace sf

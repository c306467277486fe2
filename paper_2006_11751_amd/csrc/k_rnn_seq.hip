// Recurrent cell for the few rows per time step of the learner's pass over trajectories (paper,
// Sec. 3.1: the core is unrolled over the T steps of each trajectory; hyperparameter table of
// App. "VizDoom experiments": 64 trajectories per batch).  Same arithmetic as the step's cell
// (sf_policy.h: gate rows r, z, n of a GRU; i, f, g, o of an LSTM; the incoming state zeroed
// where done is set), other work split: with 64 rows the step's kernel has 32 workgroups, each
// walking the whole K = inputs + hidden dimension in 32 dependent chunks through LDS.  Here a
// workgroup owns 32 rows x 8 hidden units, i.e. one 32 x 32 accumulator tile whose columns are
// the unit's gates ([r z n_x n_h] x 8 units, or [i f g o] x 8), its eight waves split K among
// them, and every operand goes from memory straight into the registers of the lane that feeds
// it to v_mfma_f32_32x32x2_f32: no LDS staging, all loads of a wave in flight at once.  The
// eight partial tiles meet in LDS and are added in wave order (a fixed order: results are
// reproducible), then 256 threads apply the gates.
//
// Operand order.  The MFMA takes A[i][k] from lane i + 32 k (k = 0, 1) and B[k][j] from lane
// j + 32 k.  A lane loads 16 bytes of its row at a time: lane (i, kk) loads x[i][8u + 4kk ..
// 8u + 4kk + 3] for K unit u, so MFMA e (0..3) of that unit multiplies K index 8u + 4kk + e:
// the weights are packed in that order (rnn_seq_pack), [unit group][u][lane][4 floats], one
// coalesced 16-byte load per lane and unit.  The two input pieces (FC features, encoded
// measurements) and the state follow one another in K; each is a multiple of 8 wide.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sf_internal.h"

namespace sf {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kUnits = 8;   // hidden units per workgroup

__device__ inline float sigmoid_acc(float a) { return 1.0f / (1.0f + expf(-a)); }
// (1 - e) / (1 + e) with e = exp(-2|a|), sign restored: e <= 1, nothing overflows
__device__ inline float tanh_acc(float a) {
  const float e = expf(-2.0f * fabsf(a));
  return copysignf((1.0f - e) / (1.0f + e), a);
}

struct SeqArgs {
  const void* x1;       // [B][I1] fp32, or bf16 (XB instantiations; then there is no x2)
  const float* x2;      // [B][I2] or null (I2 = 0)
  const float* h_in;    // [B][S]
  const uint8_t* done;  // [B]
  const float* wpk;     // [H / 8][(I1 + I2 + H) / 8][64][4]
  const float* b_ih;    // [G*H]
  const float* b_hh;    // [G*H]
  float* h_out;         // [B][S]
  int B, I1, I2, H;
};

// kChunk: K units (of 8) a wave has in flight per register buffer; the loop below takes two
// buffers per round, so a wave's share of K is walked in steps of 2 * kChunk units (the launch
// picks the kChunk that pads that share least).
template <bool LSTM, int kChunk, bool XB>
__global__ __launch_bounds__(kThreads, 2) void rnn_seq_kernel(SeqArgs g) {
  __shared__ float red[kWaves][16][64];  // 32 KB: the waves' partial tiles, then their sum in [0]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = LSTM ? 2 * g.H : g.H;
  const int I = g.I1 + g.I2;
  const int n_u = (I + g.H) >> 3;                 // K units in all
  const int per_wave = (n_u + kWaves - 1) / kWaves;
  const int u_begin = wave * per_wave;
  const int u_end = min(n_u, u_begin + per_wave);
  const int row0 = blockIdx.x * 32;
  // this lane's row (rows past the batch read the last row; their results are not stored)
  const int li = lane & 31, kk = lane >> 5;
  const int row = min(row0 + li, g.B - 1);
  const bool reset = g.done[row] != 0;
  const float* xr1 = (const float*)g.x1 + (size_t)row * g.I1 + 4 * kk;
  const uint16_t* xb1 = (const uint16_t*)g.x1 + (size_t)row * g.I1 + 4 * kk;
  const float* xr2 = g.x2 ? g.x2 + (size_t)row * g.I2 + 4 * kk : nullptr;
  const float* hr = g.h_in + (size_t)row * S + 4 * kk;
  const f32x4* wp = (const f32x4*)g.wpk + ((size_t)blockIdx.y * n_u) * 64 + lane;

  // The gate threads' own operands, requested ahead of the K loop: thread -> (row gi, unit gq)
  const int gi = (tid >> 3) & 31, gq = tid & 7;
  const int gm = min(row0 + gi, g.B - 1);
  const int gj = blockIdx.y * kUnits + gq;
  float bias[4], hc_prev[2];
  {
    const bool rs = g.done[gm] != 0;
    if (LSTM) {
#pragma unroll
      for (int gt = 0; gt < 4; ++gt) bias[gt] = g.b_ih[gt * g.H + gj] + g.b_hh[gt * g.H + gj];
      hc_prev[1] = g.h_in[(size_t)gm * S + g.H + gj];
      if (rs) hc_prev[1] = 0.0f;
      hc_prev[0] = 0.0f;
    } else {
      bias[0] = g.b_ih[gj] + g.b_hh[gj];
      bias[1] = g.b_ih[g.H + gj] + g.b_hh[g.H + gj];
      bias[2] = g.b_ih[2 * g.H + gj];
      bias[3] = g.b_hh[2 * g.H + gj];
      hc_prev[0] = g.h_in[(size_t)gm * S + gj];
      if (rs) hc_prev[0] = 0.0f;
      hc_prev[1] = 0.0f;
    }
  }

  // A operand of K unit u: four consecutive floats of the lane's row in the piece u falls into.
  // (Selects, not branches: a branch around a load makes the compiler wait for every load in
  // flight where the paths join.)
  auto load_a = [&](int u) -> f32x4 {
    const int k = u << 3;
    if (XB) {
      // bf16 features: both sources are read (addresses clamped into their rows), one is kept
      const uint32x2 xb = *(const uint32x2*)(xb1 + min(k, g.I1 - 8));
      f32x4 v = *(const f32x4*)(hr + max(k - I, 0));
      if (reset) v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      if (k < g.I1) {
        v[0] = __builtin_bit_cast(float, xb[0] << 16);
        v[1] = __builtin_bit_cast(float, xb[0] & 0xFFFF0000u);
        v[2] = __builtin_bit_cast(float, xb[1] << 16);
        v[3] = __builtin_bit_cast(float, xb[1] & 0xFFFF0000u);
      }
      return v;
    }
    const float* ptr = k < g.I1 ? xr1 + k : (k < I ? xr2 + (k - g.I1) : hr + (k - I));
    f32x4 v = *(const f32x4*)ptr;
    if (reset && k >= I) v = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    return v;
  };

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  f32x4 a[2][kChunk], b[2][kChunk];
  // K units u0 .. u0 + 7 of this wave; past its range the last unit's addresses (valid) are
  // read again and the weights are replaced by zeros, so that the MFMAs need no branch
  auto load_chunk = [&](int u0, f32x4 (&aa)[kChunk], f32x4 (&bb)[kChunk]) {
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      const int u = max(min(u0 + c, u_end - 1), 0);
      aa[c] = load_a(u);
      f32x4 w = wp[(size_t)u * 64];
      if (u0 + c >= u_end) w = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      bb[c] = w;
    }
  };
  auto mfma_chunk = [&](const f32x4 (&aa)[kChunk], const f32x4 (&bb)[kChunk]) {
#pragma unroll
    for (int c = 0; c < kChunk; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(aa[c][e], bb[c][e], acc, 0, 0, 0);
  };
  load_chunk(u_begin, a[0], b[0]);
  for (int u0 = u_begin; u0 < u_end; u0 += 2 * kChunk) {
    load_chunk(u0 + kChunk, a[1], b[1]);
    mfma_chunk(a[0], b[0]);
    load_chunk(u0 + 2 * kChunk, a[0], b[0]);
    mfma_chunk(a[1], b[1]);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[r];
  __syncthreads();
  // sum over the waves in wave order: two tile elements per thread
  float* flat = &red[0][0][0];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int e = tid + q * kThreads;  // [r][lane] flattened
    float s = flat[e];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) s += flat[w * 1024 + e];
    flat[e] = s;  // (element e of wave 0's tile is read by this thread only)
  }
  __syncthreads();
  // gates: tile element (i, j) is register 4*(i/8) + i%4 of lane j + 32*((i/4)%2)
  if (tid < 32 * kUnits && row0 + gi < g.B) {
    const int rr = 4 * (gi >> 3) + (gi & 3), lo = 32 * ((gi >> 2) & 1);
    float s[4];
#pragma unroll
    for (int gt = 0; gt < 4; ++gt) s[gt] = red[0][rr][lo + 8 * gt + gq];
    float* out = g.h_out + (size_t)gm * S;
    if (LSTM) {
      const float ig = sigmoid_acc(s[0] + bias[0]);
      const float fg = sigmoid_acc(s[1] + bias[1]);
      const float gg = tanh_acc(s[2] + bias[2]);
      const float og = sigmoid_acc(s[3] + bias[3]);
      const float cn = fg * hc_prev[1] + ig * gg;
      out[g.H + gj] = cn;
      out[gj] = og * tanh_acc(cn);
    } else {
      const float r = sigmoid_acc(s[0] + bias[0]);
      const float z = sigmoid_acc(s[1] + bias[1]);
      const float n = tanh_acc(s[2] + bias[2] + r * (s[3] + bias[3]));
      out[gj] = (1.0f - z) * n + z * hc_prev[0];
    }
  }
}

}  // namespace

bool rnn_seq_supported(int I1, int I2, int H) {
  return I1 > 0 && (I1 % 8) == 0 && (I2 % 8) == 0 && (H % 8) == 0;
}

// w_ih [G*H][I], w_hh [G*H][H] (values as the configuration defines them) ->
// [H / 8][(I + H) / 8][64][4]: lane (j, kk) of K unit u holds, for e = 0..3, the weight that
// multiplies K index k = 8u + 4kk + e in tile column j = 8 * gate + unit.  GRU columns: r, z
// (input and state weights), n_x (input weights, zero over the state part of K), n_h (state
// weights, zero over the input part): the n gate needs its two sums apart.
void rnn_seq_pack(const float* w_ih, const float* w_hh, int I, int H, int lstm, std::vector<float>& out) {
  const int n_u = (I + H) / 8;
  out.assign((size_t)(H / 8) * n_u * 64 * 4, 0.0f);
  for (int jb = 0; jb < H / 8; ++jb)
    for (int u = 0; u < n_u; ++u)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 4; ++e) {
          const int j = lane & 31, kk = lane >> 5;
          const int k = 8 * u + 4 * kk + e;
          const int gate = j >> 3, n = 8 * jb + (j & 7);
          float v = 0.0f;
          if (lstm || gate < 2) {
            v = k < I ? w_ih[((size_t)gate * H + n) * I + k] : w_hh[((size_t)gate * H + n) * H + (k - I)];
          } else if (gate == 2) {
            if (k < I) v = w_ih[((size_t)2 * H + n) * I + k];
          } else {
            if (k >= I) v = w_hh[((size_t)2 * H + n) * H + (k - I)];
          }
          out[(((size_t)jb * n_u + u) * 64 + lane) * 4 + e] = v;
        }
}

hipError_t launch_rnn_seq(int lstm, int B, int I1, int I2, int H, const void* x1, int x1_bf16, const float* x2,
                          const float* h_in, const uint8_t* done, const float* wpk, const float* b_ih,
                          const float* b_hh, float* h_out, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (!rnn_seq_supported(I1, x2 ? I2 : 0, H) || (x1_bf16 && x2)) return hipErrorInvalidValue;
  SeqArgs g;
  g.x1 = x1; g.x2 = x2; g.h_in = h_in; g.done = done; g.wpk = wpk; g.b_ih = b_ih; g.b_hh = b_hh;
  g.h_out = h_out; g.B = B; g.I1 = I1; g.I2 = x2 ? I2 : 0; g.H = H;
  dim3 grid((B + 31) / 32, H / kUnits);
  const int n_u = (g.I1 + g.I2 + H) / 8, per_wave = (n_u + kWaves - 1) / kWaves;
  int best = 4, best_pad = 1 << 30;
  for (int ch = 4; ch <= 9; ++ch) {
    const int pad = 2 * ch * ((per_wave + 2 * ch - 1) / (2 * ch));
    if (pad <= best_pad) {  // (ties: the larger buffer, fewer rounds)
      best_pad = pad;
      best = ch;
    }
  }
  auto go = [&](auto lstm_c, auto ch_c) {
    if (x1_bf16)
      rnn_seq_kernel<decltype(lstm_c)::value, decltype(ch_c)::value, true><<<grid, kThreads, 0, st>>>(g);
    else
      rnn_seq_kernel<decltype(lstm_c)::value, decltype(ch_c)::value, false><<<grid, kThreads, 0, st>>>(g);
  };
  auto pick = [&](auto lstm_c) {
    switch (best) {
      case 4: go(lstm_c, std::integral_constant<int, 4>{}); break;
      case 5: go(lstm_c, std::integral_constant<int, 5>{}); break;
      case 6: go(lstm_c, std::integral_constant<int, 6>{}); break;
      case 7: go(lstm_c, std::integral_constant<int, 7>{}); break;
      case 8: go(lstm_c, std::integral_constant<int, 8>{}); break;
      default: go(lstm_c, std::integral_constant<int, 9>{}); break;
    }
  };
  if (lstm) pick(std::true_type{}); else pick(std::false_type{});
  return hipGetLastError();
}

}  // namespace sf

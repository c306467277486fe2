// Recurrent core of the bf16 configurations on the 16-bit MFMA (paper, App. "Model
// architectures": LSTM core of the benchmark model, GRU cells in the large-scale runs).
//
// Same cell arithmetic, reset rule and state layout as the fp32 kernel.  The weights of a
// bf16 configuration are bf16 numbers, the core's input is a bf16 activation (rounded to
// nearest even while it is staged, or handed over as bf16 by the FC kernel, which rounds the
// same way: XB16), and the fp32 state h enters the contraction as the
// exact sum of two bf16 numbers, h = hi + lo with hi = bf16(h), lo = bf16(h - hi)
// (relative error below 2^-16): K runs over the input features and then, per 64-wide block
// of h, over its hi part and its lo part, both against the same rows of W_hh (which, like
// the block of h, are fetched once and reused from registers).  The state itself, the gates
// and the blend stay fp32.
//
// v_mfma_f32_32x32x16_bf16: lane l supplies A[i = l%32][k = 8*(l/32) + e] and
// B[k = 8*(l/32) + e][j = l%32].  The weights take the A role (i = hidden unit), the batch
// rows the B role, so a lane ends up with 4 consecutive hidden units of one batch row per
// register quad and the epilogue moves 16-byte pieces of the state.
// Workgroup: 128 batch rows (one 32-row block per wave) x 32 hidden units x all gates:
// four accumulator tiles per wave (GRU r, z, n_x, n_h; LSTM i, f, g, o).  K in chunks of 64
// through double-buffered LDS (pitch 144 bytes), global loads one chunk ahead.
#include <string.h>

#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;       // K elements per chunk
constexpr int kPitch = 144;   // LDS row pitch in bytes (128 + 16)
constexpr int kBR = 128;      // batch rows per workgroup
constexpr int kBJ = 32;       // hidden units per workgroup

// The gate functions on the hardware's exp2 and reciprocal (about 1 ulp each; no range
// reduction, no division sequence, no branches: sixteen state elements per thread pass through
// here, and with the library routines the epilogue held 40 % of the kernel's instructions).
// exp2 overflows to +inf and underflows to 0, which the reciprocal maps to 0 and 1: the
// limits come out exact.  tanh as (1 - e) / (1 + e) with e = exp(-2|a|) <= 1, sign restored.
__device__ inline float exp_hw(float a) { return __builtin_amdgcn_exp2f(a * 1.44269504088896341f); }
__device__ inline float sigmoid_acc(float a) { return __builtin_amdgcn_rcpf(1.0f + exp_hw(-a)); }
__device__ inline float tanh_acc(float a) {
  const float e = exp_hw(-2.0f * fabsf(a));
  return copysignf((1.0f - e) * __builtin_amdgcn_rcpf(1.0f + e), a);
}
__device__ inline unsigned bf16_rne(float f) {
  const unsigned u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;  // finite inputs
}
__device__ inline float bf16_value(unsigned h) { return __uint_as_float(h << 16); }

struct RnnBf16Args {
  const void* x1;         // [B][I1], fp32 or (XB16, I2 == 0) bf16
  const float* x2;        // [B][I2] or null
  const float* h_in;      // state rows of S floats, row index = batch row or ids[row]
  const uint8_t* done;    // [B]
  const uint16_t* w_ih;   // bf16 [G*H][I1 + I2]
  const uint16_t* w_hh;   // bf16 [G*H][H]
  const float* b_ih;      // [G*H]
  const float* b_hh;      // [G*H]
  float* h_out;           // [B][S]
  int B, I1, I2, H;
  const int32_t* ids;
  int n_env;
};

// 8 consecutive fp32 -> 8 bf16, round to nearest even through the packed hardware conversion:
// the values themselves (hi), and with SPLIT also what is left of them, lo = bf16(v - hi)
template <bool SPLIT>
__device__ inline void to_bf16x8(const f32x4& a, const f32x4& b, u32x4& hi_out, u32x4& lo_out) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const f32x2_t p = {v[2 * e], v[2 * e + 1]};
    const unsigned hi = __builtin_bit_cast(unsigned, __builtin_convertvector(p, bf16x2_t));
    hi_out[e] = hi;
    if (SPLIT) {
      const f32x2_t r = {v[2 * e] - __uint_as_float(hi << 16), v[2 * e + 1] - __uint_as_float(hi & 0xFFFF0000u)};
      lo_out[e] = __builtin_bit_cast(unsigned, __builtin_convertvector(r, bf16x2_t));
    }
  }
}

template <bool LSTM, bool XB16>
__global__ __launch_bounds__(256) void rnn_bf16_kernel(RnnBf16Args g) {
  constexpr int NG = LSTM ? 4 : 3;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * (kBR + NG * kBJ) * kPitch];
  unsigned char* Rs = smem;                       // [2][128][pitch] batch rows
  unsigned char* Ws = smem + 2 * kBR * kPitch;    // [2][NG*32][pitch] weight rows

  const int B = g.B, H = g.H, I = g.I1 + g.I2;
  const int S = LSTM ? 2 * H : H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.x * kBR, j0 = blockIdx.y * kBJ;
  const int lrow = tid >> 3, lk8 = (tid & 7) * 8;  // 8 threads x 8 elements per tile row

  int am[4], ah[4];
  bool areset[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int m = m0 + lrow + 32 * r;
    am[r] = m < B ? m : B - 1;  // rows past the end re-read the last row; never stored
    areset[r] = g.done[am[r]] != 0;
    ah[r] = am[r];
    if (g.ids) {
      const int e = g.ids[am[r]];
      const bool ok = (unsigned)e < (unsigned)g.n_env;
      ah[r] = ok ? e : 0;
      areset[r] = areset[r] || !ok;
    }
  }
  const int n1c = g.I1 / kBK, nxc = I / kBK, nhc = H / kBK;

  f32x4 ra[4][2];
  u32x4 rw[NG];
  // K runs over the x chunks and then, per 64-wide block of h, over its hi part and its lo
  // part: the lo chunk reuses the state values and the weight rows that the hi chunk loaded
  // (they stay in registers), so every block of h and of W_hh is fetched once.
  auto gload_x = [&](int c) {
    const int kk = c * kBK + lk8;
    if (XB16) {  // eight bf16 values, kept as they are in the first register quad
#pragma unroll
      for (int r = 0; r < 4; ++r)
        ra[r][0] = *(const f32x4*)((const uint16_t*)g.x1 + (size_t)am[r] * g.I1 + kk);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float* src = c < n1c ? (const float*)g.x1 + (size_t)am[r] * g.I1 + kk
                                   : g.x2 + (size_t)am[r] * g.I2 + (kk - g.I1);
        ra[r][0] = *(const f32x4*)src;
        ra[r][1] = *(const f32x4*)(src + 4);
      }
    }
#pragma unroll
    for (int q = 0; q < NG; ++q)
      rw[q] = *(const u32x4*)(g.w_ih + (size_t)(q * H + j0 + lrow) * I + kk);
  };
  auto gload_h = [&](int kb) {
    const int kk = kb * kBK + lk8;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float* src = g.h_in + (size_t)ah[r] * S + kk;
      ra[r][0] = *(const f32x4*)src;
      ra[r][1] = *(const f32x4*)(src + 4);
    }
#pragma unroll
    for (int q = 0; q < NG; ++q)
      rw[q] = *(const u32x4*)(g.w_hh + (size_t)(q * H + j0 + lrow) * H + kk);
  };
  // rphase: 0 = x values, 1 = hi parts of h, 2 = lo parts of h.  A block of h is split once,
  // when its hi part is stored: the lo words then take the place of the fp32 values in the
  // registers and phase 2 only stores them.
  auto sstore = [&](int buf, int rphase) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      // the reset is applied here, not behind the load (a select there waits for the load)
      const u32x4 zero = {0u, 0u, 0u, 0u};
      u32x4 v, lo;
      if (rphase == 0) {
        if (XB16) v = __builtin_bit_cast(u32x4, ra[r][0]);
        else to_bf16x8<false>(ra[r][0], ra[r][1], v, lo);
      } else if (rphase == 1) {
        to_bf16x8<true>(ra[r][0], ra[r][1], v, lo);
        ra[r][0] = __builtin_bit_cast(f32x4, lo);
      } else {
        v = __builtin_bit_cast(u32x4, ra[r][0]);
      }
      *(u32x4*)(Rs + (buf * kBR + lrow + 32 * r) * kPitch + lk8 * 2) = (rphase != 0 && areset[r]) ? zero : v;
    }
#pragma unroll
    for (int q = 0; q < NG; ++q)
      *(u32x4*)(Ws + (buf * NG * kBJ + q * kBJ + lrow) * kPitch + lk8 * 2) = rw[q];
  };

  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

  auto compute = [&](int buf, auto xph) {
    const unsigned char* rb = Rs + (buf * kBR + wave * 32 + li) * kPitch + lh * 16;
    const unsigned char* wb = Ws + (buf * NG * kBJ + li) * kPitch + lh * 16;
    constexpr bool xphase = decltype(xph)::value;
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      const bf16x8 bfrag = __builtin_bit_cast(bf16x8, *(const u32x4*)(rb + ks * 32));
      bf16x8 afrag[NG];
#pragma unroll
      for (int q = 0; q < NG; ++q)
        afrag[q] = __builtin_bit_cast(bf16x8, *(const u32x4*)(wb + q * kBJ * kPitch + ks * 32));
      if (LSTM) {
#pragma unroll
        for (int q = 0; q < NG; ++q)
          acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[q], bfrag, acc[q], 0, 0, 0);
      } else {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[0], bfrag, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[1], bfrag, acc[1], 0, 0, 0);
        if (xphase)
          acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[2], bfrag, acc[2], 0, 0, 0);
        else
          acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[2], bfrag, acc[3], 0, 0, 0);
      }
    }
  };

  // Single register set: loads of the next chunk, MFMAs of this one, conversion and LDS
  // store of the next, barrier; `cb` counts chunks (LDS buffer = parity).  One plain loop
  // per accumulator set, no conditions around the loads.
  using Xp = std::true_type;
  using Hp = std::false_type;
  int cb = 0;
  gload_x(0);
  sstore(0, 0);
  __syncthreads();
  for (int c = 0; c + 1 < nxc; ++c, ++cb) {
    gload_x(c + 1);
    compute(cb & 1, Xp{});
    sstore((cb + 1) & 1, 0);
    __syncthreads();
  }
  gload_h(0);  // the last x chunk runs while block 0 of h arrives
  compute(cb & 1, Xp{});
  sstore((cb + 1) & 1, 1);
  __syncthreads();
  ++cb;
  for (int kb = 0; kb + 1 < nhc; ++kb) {
    compute(cb & 1, Hp{});      // hi part of block kb
    sstore((cb + 1) & 1, 2);    // its lo part, from the same registers
    __syncthreads();
    ++cb;
    gload_h(kb + 1);
    compute(cb & 1, Hp{});      // lo part of block kb
    sstore((cb + 1) & 1, 1);    // hi part of block kb + 1
    __syncthreads();
    ++cb;
  }
  compute(cb & 1, Hp{});
  sstore((cb + 1) & 1, 2);
  __syncthreads();
  ++cb;
  compute(cb & 1, Hp{});

  // epilogue: register 4*q4 + u of a tile holds hidden unit j0 + 8*q4 + 4*lh + u of batch
  // row m0 + wave*32 + li
  const int m = m0 + wave * 32 + li;
  if (m >= B) return;
  int hm = m;
  bool reset = g.done[m] != 0;
  if (g.ids) {
    const int e = g.ids[m];
    const bool ok = (unsigned)e < (unsigned)g.n_env;
    hm = ok ? e : 0;
    reset = reset || !ok;
  }
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const int j = j0 + 8 * q4 + 4 * lh;
    f32x4 bi[NG], bh[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) {
      bi[q] = *(const f32x4*)(g.b_ih + q * H + j);
      bh[q] = *(const f32x4*)(g.b_hh + q * H + j);
    }
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    if (LSTM) {
      const f32x4 cprev = reset ? zero : *(const f32x4*)(g.h_in + (size_t)hm * S + H + j);
      f32x4 hn, cn;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float ig = sigmoid_acc(acc[0][4 * q4 + u] + bi[0][u] + bh[0][u]);
        const float fg = sigmoid_acc(acc[1][4 * q4 + u] + bi[1][u] + bh[1][u]);
        const float gg = tanh_acc(acc[2][4 * q4 + u] + bi[2][u] + bh[2][u]);
        const float og = sigmoid_acc(acc[3][4 * q4 + u] + bi[NG - 1][u] + bh[NG - 1][u]);
        cn[u] = fg * cprev[u] + ig * gg;
        hn[u] = og * tanh_acc(cn[u]);
      }
      *(f32x4*)(g.h_out + (size_t)m * S + H + j) = cn;
      *(f32x4*)(g.h_out + (size_t)m * S + j) = hn;
    } else {
      const f32x4 hprev = reset ? zero : *(const f32x4*)(g.h_in + (size_t)hm * S + j);
      f32x4 hn;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float r = sigmoid_acc(acc[0][4 * q4 + u] + bi[0][u] + bh[0][u]);
        const float z = sigmoid_acc(acc[1][4 * q4 + u] + bi[1][u] + bh[1][u]);
        const float n = tanh_acc(acc[2][4 * q4 + u] + bi[2][u] + r * (acc[3][4 * q4 + u] + bh[2][u]));
        hn[u] = (1.0f - z) * n + z * hprev[u];
      }
      *(f32x4*)(g.h_out + (size_t)m * S + j) = hn;
    }
  }
}

}  // namespace

// Every piece of the input and the state width must be whole 64-wide K chunks.
bool rnn_bf16_supported(int I1, int I2, int H) {
  return I1 > 0 && (I1 % kBK) == 0 && (I2 % kBK) == 0 && (H % kBK) == 0;
}

// bf16 bits of weights that are bf16 numbers already (rounded to nearest even otherwise)
void rnn_bf16_pack(const float* w, size_t n, std::vector<uint16_t>& out) {
  out.resize(n);
  for (size_t i = 0; i < n; ++i) {
    uint32_t u;
    memcpy(&u, &w[i], 4);
    out[i] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
  }
}

// x1_bf16: x1 holds bf16 values (only without a second input)
hipError_t launch_rnn_bf16(int lstm, int B, int I1, int I2, int H, const void* x1, int x1_bf16,
                           const float* x2, const float* h_in, const uint8_t* done,
                           const uint16_t* w_ih, const uint16_t* w_hh, const float* b_ih,
                           const float* b_hh, float* h_out, const int32_t* ids, int n_env,
                           hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (x1_bf16 && x2) return hipErrorInvalidValue;
  RnnBf16Args g;
  g.x1 = x1; g.x2 = x2; g.h_in = h_in; g.done = done;
  g.w_ih = w_ih; g.w_hh = w_hh; g.b_ih = b_ih; g.b_hh = b_hh; g.h_out = h_out;
  g.B = B; g.I1 = I1; g.I2 = x2 ? I2 : 0; g.H = H; g.ids = ids; g.n_env = n_env;
  dim3 grid((B + kBR - 1) / kBR, H / kBJ);
  if (lstm) {
    if (x1_bf16) rnn_bf16_kernel<true, true><<<grid, 256, 0, st>>>(g);
    else rnn_bf16_kernel<true, false><<<grid, 256, 0, st>>>(g);
  } else {
    if (x1_bf16) rnn_bf16_kernel<false, true><<<grid, 256, 0, st>>>(g);
    else rnn_bf16_kernel<false, false><<<grid, 256, 0, st>>>(g);
  }
  return hipGetLastError();
}

}  // namespace sf

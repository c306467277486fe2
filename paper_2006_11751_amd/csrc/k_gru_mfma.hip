// GRU cell with the episode-boundary reset, gate GEMMs on the fp32 MFMA and the
// gate arithmetic fused into the epilogue (paper, App. "Model architectures": RNN
// core; GRU cells in the large-scale experiments).
//
//   h  = done ? 0 : h_in
//   r  = sigmoid(W_ir x + b_ir + W_hr h + b_hr)
//   z  = sigmoid(W_iz x + b_iz + W_hz h + b_hz)
//   n  = tanh   (W_in x + b_in + r * (W_hn h + b_hn))
//   h' = (1 - z) * n + z * h
//
// A workgroup owns 64 batch rows x 32 hidden units and keeps four accumulator tiles
// per 32x32 block: r and z (summed over x and h), n_x (x part) and n_h (h part,
// which the reset gate multiplies).  K runs over the input features (weights W_ih)
// and then over the previous state (weights W_hh): three MFMAs per K step in either
// phase, sharing the A fragment.  Waves are arranged 2 (rows) x 2 (K split inside
// each 32-wide chunk); the partial tiles are summed through LDS in a fixed order and
// the wave that holds the sum applies the gates and writes h_out once.
// Operand staging, LDS pitch and the K-to-lane mapping are those of the GEMM kernel.
#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;
constexpr int kPitch = 36;
constexpr int kBM = 64;   // batch rows per workgroup
constexpr int kBJ = 32;   // hidden units per workgroup

__device__ inline float sigmoid_acc(float a) { return 1.0f / (1.0f + expf(-a)); }

__global__ __launch_bounds__(256) void gru_mfma_kernel(
    const float* __restrict__ x, const float* __restrict__ h_in, const uint8_t* __restrict__ done,
    const float* __restrict__ w_ih, const float* __restrict__ w_hh,
    const float* __restrict__ b_ih, const float* __restrict__ b_hh, float* __restrict__ h_out,
    int B, int I, int H) {
  __shared__ float smem[2 * (kBM + 3 * kBJ) * kPitch];
  float* As = smem;                       // [2][64][pitch]
  float* Bs = smem + 2 * kBM * kPitch;    // [2][96][pitch]  rows: r(32), z(32), n(32)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wk = wave >> 1;
  const int li = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.x * kBM, j0 = blockIdx.y * kBJ;
  const int lrow = tid >> 3, lk4 = (tid & 7) * 4;

  // A rows (2 per thread) and B rows (3 per thread: one per gate)
  int am[2];
  bool areset[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    int m = m0 + lrow + 32 * r;
    am[r] = m < B ? m : B - 1;
    areset[r] = done[am[r]] != 0;
  }
  f32x4 ra[2], rb[3];
  const int nx_chunks = I / kBK, nchunks = nx_chunks + H / kBK;
  auto gload = [&](int c) {
    if (c < nx_chunks) {
      const int kk = c * kBK + lk4;
#pragma unroll
      for (int r = 0; r < 2; ++r) ra[r] = *(const f32x4*)(x + (size_t)am[r] * I + kk);
#pragma unroll
      for (int q = 0; q < 3; ++q) rb[q] = *(const f32x4*)(w_ih + (size_t)(q * H + j0 + lrow) * I + kk);
    } else {
      const int kk = (c - nx_chunks) * kBK + lk4;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        f32x4 v = *(const f32x4*)(h_in + (size_t)am[r] * H + kk);
        const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
        ra[r] = areset[r] ? zero : v;
      }
#pragma unroll
      for (int q = 0; q < 3; ++q) rb[q] = *(const f32x4*)(w_hh + (size_t)(q * H + j0 + lrow) * H + kk);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int r = 0; r < 2; ++r) *(f32x4*)&As[(buf * kBM + lrow + 32 * r) * kPitch + lk4] = ra[r];
#pragma unroll
    for (int q = 0; q < 3; ++q) *(f32x4*)&Bs[(buf * 3 * kBJ + q * kBJ + lrow) * kPitch + lk4] = rb[q];
  };

  f32x16 acc_r, acc_z, acc_nx, acc_nh;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_r[v] = acc_z[v] = acc_nx[v] = acc_nh[v] = 0.0f;

  gload(0);
  sstore(0);
  __syncthreads();
  for (int c = 0; c < nchunks; ++c) {
    const int buf = c & 1;
    if (c + 1 < nchunks) gload(c + 1);
    const float* Ab = As + (buf * kBM + wm * 32 + li) * kPitch + 4 * lh;
    const float* Bb = Bs + (buf * 3 * kBJ + li) * kPitch + 4 * lh;
    const bool xphase = c < nx_chunks;
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
      const int kg = (gi * 2 + wk) * 8;
      const f32x4 af = *(const f32x4*)(Ab + kg);
      const f32x4 br = *(const f32x4*)(Bb + kg);
      const f32x4 bz = *(const f32x4*)(Bb + kBJ * kPitch + kg);
      const f32x4 bn = *(const f32x4*)(Bb + 2 * kBJ * kPitch + kg);
      if (xphase) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          acc_r = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], br[t], acc_r, 0, 0, 0);
          acc_z = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bz[t], acc_z, 0, 0, 0);
          acc_nx = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bn[t], acc_nx, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          acc_r = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], br[t], acc_r, 0, 0, 0);
          acc_z = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bz[t], acc_z, 0, 0, 0);
          acc_nh = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bn[t], acc_nh, 0, 0, 0);
        }
      }
    }
    if (c + 1 < nchunks) sstore(buf ^ 1);
    __syncthreads();
  }

  // K-split reduction: wk = 1 hands its four tiles to wk = 0 through LDS
  float* red = smem + wm * (4 * 16 * 64);
  if (wk == 1) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      red[(0 * 16 + v) * 64 + lane] = acc_r[v];
      red[(1 * 16 + v) * 64 + lane] = acc_z[v];
      red[(2 * 16 + v) * 64 + lane] = acc_nx[v];
      red[(3 * 16 + v) * 64 + lane] = acc_nh[v];
    }
  }
  __syncthreads();
  if (wk != 0) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    acc_r[v] += red[(0 * 16 + v) * 64 + lane];
    acc_z[v] += red[(1 * 16 + v) * 64 + lane];
    acc_nx[v] += red[(2 * 16 + v) * 64 + lane];
    acc_nh[v] += red[(3 * 16 + v) * 64 + lane];
  }

  // gates; tile element (v, lane): row i = (v%4) + 4*(lane/32) + 8*(v/4), column j = lane%32
  const int j = j0 + li;
  const float bir = b_ih[j] + b_hh[j], biz = b_ih[H + j] + b_hh[H + j];
  const float bin = b_ih[2 * H + j], bhn = b_hh[2 * H + j];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + wm * 32 + (v & 3) + 4 * lh + 8 * (v >> 2);
    if (m < B) {
      const float hprev = done[m] ? 0.0f : h_in[(size_t)m * H + j];
      const float r = sigmoid_acc(acc_r[v] + bir);
      const float z = sigmoid_acc(acc_z[v] + biz);
      const float n = tanhf(acc_nx[v] + bin + r * (acc_nh[v] + bhn));
      h_out[(size_t)m * H + j] = (1.0f - z) * n + z * hprev;
    }
  }
}

}  // namespace

bool gru_mfma_supported(int I, int H) { return (I % kBK) == 0 && (H % kBK) == 0; }

hipError_t launch_gru_mfma(int B, int I, int H, const float* x, const float* h_in,
                           const uint8_t* done, const float* w_ih, const float* w_hh,
                           const float* b_ih, const float* b_hh, float* h_out, hipStream_t st) {
  if (B == 0) return hipSuccess;
  dim3 grid((B + kBM - 1) / kBM, H / kBJ);
  gru_mfma_kernel<<<grid, 256, 0, st>>>(x, h_in, done, w_ih, w_hh, b_ih, b_hh, h_out, B, I, H);
  return hipGetLastError();
}

}  // namespace sf

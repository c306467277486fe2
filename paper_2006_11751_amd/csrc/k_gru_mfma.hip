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
// A workgroup owns BM batch rows x 32 hidden units and keeps four accumulator tiles
// per 32x32 block: r and z (summed over x and h), n_x (x part) and n_h (h part,
// which the reset gate multiplies).  K runs over the input features (weights W_ih)
// and then over the previous state (weights W_hh): three MFMAs per K step in either
// phase, sharing the A fragment.  The four waves are arranged WM (rows) x WK (K
// split inside each 32-wide chunk): BM = 32 uses a four-way split, which doubles the
// number of workgroups for small batches.  Every wave writes its partial tiles to
// LDS; after one barrier wave wk of a row block sums the partials (fixed order) for
// its 16/WK share of the tile rows, applies the gates and writes h_out once.
// Operand staging (two register sets, global loads two chunks ahead), LDS pitch and
// the K-to-lane mapping are those of the GEMM kernel.
#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;
constexpr int kP = 36;    // LDS row pitch (floats)
constexpr int kBJ = 32;   // hidden units per workgroup
constexpr int kRedFloats = 4 * 4 * 16 * 64;  // [wave][tile][v][lane]

__device__ inline float sigmoid_acc(float a) { return 1.0f / (1.0f + expf(-a)); }

template <int BM>
__global__ __launch_bounds__(256) void gru_mfma_kernel(
    const float* __restrict__ x, const float* __restrict__ h_in, const uint8_t* __restrict__ done,
    const float* __restrict__ w_ih, const float* __restrict__ w_hh,
    const float* __restrict__ b_ih, const float* __restrict__ b_hh, float* __restrict__ h_out,
    int B, int I, int H, const int32_t* __restrict__ ids, int n_env) {
  constexpr int WM = BM / 32, WK = 4 / WM;
  constexpr int RA = BM / 32;       // 16-byte A loads per thread per chunk (B: 3, one per gate)
  constexpr int GPW = 4 / WK;       // K groups per wave per chunk
  constexpr int TILE_FLOATS = 2 * (BM + 3 * kBJ) * kP;
  __shared__ float smem[TILE_FLOATS > kRedFloats ? TILE_FLOATS : kRedFloats];
  float* As = smem;                     // [2][BM][pitch]
  float* Bs = smem + 2 * BM * kP;       // [2][96][pitch]  rows: r(32), z(32), n(32)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wk = wave / WM;
  const int li = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.x * BM, j0 = blockIdx.y * kBJ;
  const int lrow = tid >> 3, lk4 = (tid & 7) * 4;

  // With ids, row m's state is row ids[m] of a table of n_env rows; an id outside the table
  // reads as a zero state.
  int am[RA], ah[RA];
  bool areset[RA];
#pragma unroll
  for (int r = 0; r < RA; ++r) {
    int m = m0 + lrow + 32 * r;
    am[r] = m < B ? m : B - 1;  // rows past the end re-read the last row; never stored
    areset[r] = done[am[r]] != 0;
    ah[r] = am[r];
    if (ids) {
      const int e = ids[am[r]];
      const bool ok = (unsigned)e < (unsigned)n_env;
      ah[r] = ok ? e : 0;
      areset[r] = areset[r] || !ok;
    }
  }
  f32x4 ra[2][RA], rb[2][3];
  const int nx_chunks = I / kBK, nchunks = nx_chunks + H / kBK;
  auto gload = [&](auto set, int c) {
    constexpr int S = decltype(set)::value;
    if (c < nx_chunks) {
      const int kk = c * kBK + lk4;
#pragma unroll
      for (int r = 0; r < RA; ++r) ra[S][r] = *(const f32x4*)(x + (size_t)am[r] * I + kk);
#pragma unroll
      for (int q = 0; q < 3; ++q)
        rb[S][q] = *(const f32x4*)(w_ih + (size_t)(q * H + j0 + lrow) * I + kk);
    } else {
      const int kk = (c - nx_chunks) * kBK + lk4;
#pragma unroll
      for (int r = 0; r < RA; ++r) {
        const f32x4 v = *(const f32x4*)(h_in + (size_t)ah[r] * H + kk);
        const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
        ra[S][r] = areset[r] ? zero : v;
      }
#pragma unroll
      for (int q = 0; q < 3; ++q)
        rb[S][q] = *(const f32x4*)(w_hh + (size_t)(q * H + j0 + lrow) * H + kk);
    }
  };
  auto sstore = [&](auto set, int buf) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int r = 0; r < RA; ++r) *(f32x4*)&As[(buf * BM + lrow + 32 * r) * kP + lk4] = ra[S][r];
#pragma unroll
    for (int q = 0; q < 3; ++q)
      *(f32x4*)&Bs[(buf * 3 * kBJ + q * kBJ + lrow) * kP + lk4] = rb[S][q];
  };

  f32x16 acc_r, acc_z, acc_nx, acc_nh;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_r[v] = acc_z[v] = acc_nx[v] = acc_nh[v] = 0.0f;

  auto compute = [&](int c) {
    const int buf = c & 1;
    const float* Ab = As + (buf * BM + wm * 32 + li) * kP + 4 * lh;
    const float* Bb = Bs + (buf * 3 * kBJ + li) * kP + 4 * lh;
    const bool xphase = c < nx_chunks;
#pragma unroll
    for (int gi = 0; gi < GPW; ++gi) {
      const int kg = (gi * WK + wk) * 8;
      const f32x4 af = *(const f32x4*)(Ab + kg);
      const f32x4 br = *(const f32x4*)(Bb + kg);
      const f32x4 bz = *(const f32x4*)(Bb + kBJ * kP + kg);
      const f32x4 bn = *(const f32x4*)(Bb + 2 * kBJ * kP + kg);
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
  };
  auto step = [&](auto set, int c) {
    constexpr int S = decltype(set)::value;
    if (c + 2 < nchunks) gload(set, c + 2);
    compute(c);
    if (c + 1 < nchunks) sstore(std::integral_constant<int, S ^ 1>{}, (c + 1) & 1);
    __syncthreads();
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  gload(I0{}, 0);
  sstore(I0{}, 0);
  if (nchunks > 1) gload(I1{}, 1);
  __syncthreads();
  for (int c = 0; c < nchunks; c += 2) {
    step(I0{}, c);
    if (c + 1 < nchunks) step(I1{}, c + 1);
  }

  // partial tiles of every wave -> LDS (the tile buffers are no longer read)
  float* red = smem;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    red[((wave * 4 + 0) * 16 + v) * 64 + lane] = acc_r[v];
    red[((wave * 4 + 1) * 16 + v) * 64 + lane] = acc_z[v];
    red[((wave * 4 + 2) * 16 + v) * 64 + lane] = acc_nx[v];
    red[((wave * 4 + 3) * 16 + v) * 64 + lane] = acc_nh[v];
  }
  __syncthreads();

  // wave wk finishes tile rows v in [wk*16/WK, (wk+1)*16/WK): sum over the K split in
  // the order k-split 0, 1, ..., then gates.  Tile element (v, lane): row
  // i = (v%4) + 4*(lane/32) + 8*(v/4), column j = lane%32.
  const int j = j0 + li;
  const float bir = b_ih[j] + b_hh[j], biz = b_ih[H + j] + b_hh[H + j];
  const float bin = b_ih[2 * H + j], bhn = b_hh[2 * H + j];
  constexpr int VPW = 16 / WK;
#pragma unroll
  for (int u = 0; u < VPW; ++u) {
    const int v = wk * VPW + u;
    float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int k = 0; k < WK; ++k) {
      const int src = wm + WM * k;  // wave index holding k-split k of this row block
#pragma unroll
      for (int t = 0; t < 4; ++t) s[t] += red[((src * 4 + t) * 16 + v) * 64 + lane];
    }
    const int m = m0 + wm * 32 + (v & 3) + 4 * lh + 8 * (v >> 2);
    if (m < B) {
      int hm = m;
      bool reset = done[m] != 0;
      if (ids) {
        const int e = ids[m];
        const bool ok = (unsigned)e < (unsigned)n_env;
        hm = ok ? e : 0;
        reset = reset || !ok;
      }
      const float hprev = reset ? 0.0f : h_in[(size_t)hm * H + j];
      const float r = sigmoid_acc(s[0] + bir);
      const float z = sigmoid_acc(s[1] + biz);
      const float n = tanhf(s[2] + bin + r * (s[3] + bhn));
      h_out[(size_t)m * H + j] = (1.0f - z) * n + z * hprev;
    }
  }
}

}  // namespace

bool gru_mfma_supported(int I, int H) { return (I % kBK) == 0 && (H % kBK) == 0; }

// Row-block size: 64 rows per workgroup when that still gives every CU several
// workgroups, else 32.  Callers fix the choice once, from the largest batch.
int gru_mfma_pick_bm(int max_batch, int H) {
  long long wgs64 = (long long)((max_batch + 63) / 64) * (H / kBJ);
  return wgs64 >= 1024 ? 64 : 32;
}

hipError_t launch_gru_mfma(int B, int I, int H, const float* x, const float* h_in,
                           const uint8_t* done, const float* w_ih, const float* w_hh,
                           const float* b_ih, const float* b_hh, float* h_out, int bm,
                           const int32_t* ids, int n_env, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (bm == 64) {
    dim3 grid((B + 63) / 64, H / kBJ);
    gru_mfma_kernel<64><<<grid, 256, 0, st>>>(x, h_in, done, w_ih, w_hh, b_ih, b_hh, h_out, B, I, H,
                                                  ids, n_env);
  } else {
    dim3 grid((B + 31) / 32, H / kBJ);
    gru_mfma_kernel<32><<<grid, 256, 0, st>>>(x, h_in, done, w_ih, w_hh, b_ih, b_hh, h_out, B, I, H,
                                                  ids, n_env);
  }
  return hipGetLastError();
}

}  // namespace sf

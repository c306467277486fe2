// Recurrent core with the episode-boundary reset: gate GEMMs on the fp32 MFMA and the gate
// arithmetic fused into the epilogue (paper, App. "Model architectures": the benchmark
// model's core is an LSTM; GRU cells in the large-scale experiments).
//
//   state after the reset:  h = done ? 0 : h_in   (LSTM: c likewise)
//   GRU    r  = sigmoid(W_ir x + b_ir + W_hr h + b_hr)
//          z  = sigmoid(W_iz x + b_iz + W_hz h + b_hz)
//          n  = tanh   (W_in x + b_in + r * (W_hn h + b_hn))
//          h' = (1 - z) * n + z * h
//   LSTM   i, f, o = sigmoid(W_i* x + b_i* + W_h* h + b_h*),  g = tanh(W_ig x + b_ig + W_hg h + b_hg)
//          c' = f * c + i * g,   h' = o * tanh(c')
//   A state row holds rnn_dim floats (GRU) or [h | c] (LSTM).
//
// A workgroup owns BM batch rows x 32 hidden units and keeps four accumulator tiles per
// 32x32 block.  GRU: r and z (summed over x and h), n_x (x part) and n_h (h part, which the
// reset gate multiplies): three MFMAs per K step.  LSTM: i, f, g, o, each summed over x
// and h: four MFMAs per K step.  K runs over the input features (weights W_ih) and then
// over the previous h (weights W_hh); the input features may come in two pieces (the
// encoder's features and the encoded measurement vector of the full architecture), which
// stand side by side in W_ih's columns.  The four waves are arranged WM (rows) x WK (K
// split inside each 32-wide chunk): BM = 32 uses a four-way split, which doubles the
// number of workgroups for small batches.  Every wave writes its partial tiles to LDS;
// after one barrier wave wk of a row block sums the partials (fixed order) for its 16/WK
// share of the tile rows, applies the gates and writes the new state once.
// Operand staging (two register sets, global loads two chunks ahead), LDS pitch and the
// K-to-lane mapping are those of the GEMM kernel.
#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;
constexpr int kP = 36;    // LDS row pitch (floats)
constexpr int kBJ = 32;   // hidden units per workgroup
constexpr int kRedFloats = 4 * 2 * 16 * 64;  // [wave][tile of a pair][v][lane]: 32 KB, below the operand tiles

__device__ inline float sigmoid_acc(float a) { return 1.0f / (1.0f + expf(-a)); }
// tanh without the library routine's branches: (1 - e) / (1 + e) with e = exp(-2|a|), sign
// restored; e <= 1, so nothing overflows, and the error stays at a few ulp
__device__ inline float tanh_acc(float a) {
  const float e = expf(-2.0f * fabsf(a));
  return copysignf((1.0f - e) / (1.0f + e), a);
}

struct RnnArgs {
  const float* x1;      // [B][I1]
  const float* x2;      // [B][I2] or null (I2 = 0)
  const float* h_in;    // state rows of S floats, row index = batch row or ids[row]
  const uint8_t* done;  // [B]
  const float* w_ih;    // [G*H][I1 + I2]
  const float* w_hh;    // [G*H][H]
  const float* b_ih;    // [G*H]
  const float* b_hh;    // [G*H]
  float* h_out;         // [B][S]
  int B, I1, I2, H;
  const int32_t* ids;   // [B] or null
  int n_env;
};

// PAIRS (GRU only): the x chunks and the h chunks both come in pairs (I1 + I2 and H multiples
// of 64), which lets the K loop be written as two plain loops, one per accumulator set.
template <int BM, bool LSTM, bool PAIRS>
__global__ __launch_bounds__(256, (BM == 32 && !LSTM && PAIRS) ? 3 : 1) void rnn_mfma_kernel(RnnArgs g) {
  constexpr int NG = LSTM ? 4 : 3;  // gate blocks of the weight matrices
  constexpr int WM = BM / 32, WK = 4 / WM;
  constexpr int RA = BM / 32;       // 16-byte A loads per thread per chunk (B: one per gate)
  constexpr int GPW = 4 / WK;       // K groups per wave per chunk
  constexpr int TILE_FLOATS = 2 * (BM + NG * kBJ) * kP;
  __shared__ float smem[TILE_FLOATS > kRedFloats ? TILE_FLOATS : kRedFloats];
  float* As = smem;                     // [2][BM][pitch]
  float* Bs = smem + 2 * BM * kP;       // [2][NG*32][pitch]  rows: one block of 32 per gate

  const int B = g.B, H = g.H, I = g.I1 + g.I2;
  const int S = LSTM ? 2 * H : H;       // floats per state row
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
    areset[r] = g.done[am[r]] != 0;
    ah[r] = am[r];
    if (g.ids) {
      const int e = g.ids[am[r]];
      const bool ok = (unsigned)e < (unsigned)g.n_env;
      ah[r] = ok ? e : 0;
      areset[r] = areset[r] || !ok;
    }
  }
  f32x4 ra[2][RA], rb[2][NG];
  const int n1_chunks = g.I1 / kBK, nx_chunks = I / kBK, nchunks = nx_chunks + H / kBK;
  // The reset (state rows of finished episodes read as zero) is applied when a set moves to
  // LDS, not when it is loaded: a select right behind the load would wait for it there and
  // then, with every other load of the prefetch.
  bool set_is_h[2] = {false, false};
  auto gload = [&](auto set, int c) {
    constexpr int SET = decltype(set)::value;
    set_is_h[SET] = c >= nx_chunks;
    if (c < nx_chunks) {
      const int kk = c * kBK + lk4;  // column of W_ih
      if (c < n1_chunks) {
#pragma unroll
        for (int r = 0; r < RA; ++r) ra[SET][r] = *(const f32x4*)(g.x1 + (size_t)am[r] * g.I1 + kk);
      } else {
#pragma unroll
        for (int r = 0; r < RA; ++r)
          ra[SET][r] = *(const f32x4*)(g.x2 + (size_t)am[r] * g.I2 + (kk - g.I1));
      }
#pragma unroll
      for (int q = 0; q < NG; ++q)
        rb[SET][q] = *(const f32x4*)(g.w_ih + (size_t)(q * H + j0 + lrow) * I + kk);
    } else {
      const int kk = (c - nx_chunks) * kBK + lk4;
#pragma unroll
      for (int r = 0; r < RA; ++r) ra[SET][r] = *(const f32x4*)(g.h_in + (size_t)ah[r] * S + kk);
#pragma unroll
      for (int q = 0; q < NG; ++q)
        rb[SET][q] = *(const f32x4*)(g.w_hh + (size_t)(q * H + j0 + lrow) * H + kk);
    }
  };
  auto sstore = [&](auto set, int buf) {
    constexpr int SET = decltype(set)::value;
#pragma unroll
    for (int r = 0; r < RA; ++r) {
      const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
      *(f32x4*)&As[(buf * BM + lrow + 32 * r) * kP + lk4] = (set_is_h[SET] && areset[r]) ? zero : ra[SET][r];
    }
#pragma unroll
    for (int q = 0; q < NG; ++q)
      *(f32x4*)&Bs[(buf * NG * kBJ + q * kBJ + lrow) * kP + lk4] = rb[SET][q];
  };

  // What the gate epilogue needs from memory is fetched before the K loop (biases, the
  // previous state of this thread's outputs): after the loop each of these loads would add
  // its latency to every workgroup, and in a one-round grid nothing else hides it.
  // Wave wk finishes tile rows v in [wk*16/WK, (wk+1)*16/WK); tile element (v, lane) is row
  // i = (v%4) + 4*(lane/32) + 8*(v/4), column j = lane%32.
  constexpr int VPW = 16 / WK;
  const int j = j0 + li;
  float bias[4];
  if (LSTM) {
#pragma unroll
    for (int q = 0; q < 4; ++q) bias[q] = g.b_ih[q * H + j] + g.b_hh[q * H + j];
  } else {
    bias[0] = g.b_ih[j] + g.b_hh[j];
    bias[1] = g.b_ih[H + j] + g.b_hh[H + j];
    bias[2] = g.b_ih[2 * H + j];
    bias[3] = g.b_hh[2 * H + j];
  }
  float sprev[VPW];  // GRU: previous h; LSTM: previous c (zero after a reset)
#pragma unroll
  for (int u = 0; u < VPW; ++u) {
    const int v = wk * VPW + u;
    int m = m0 + wm * 32 + (v & 3) + 4 * lh + 8 * (v >> 2);
    m = m < B ? m : B - 1;
    int hm = m;
    bool reset = g.done[m] != 0;
    if (g.ids) {
      const int e = g.ids[m];
      const bool ok = (unsigned)e < (unsigned)g.n_env;
      hm = ok ? e : 0;
      reset = reset || !ok;
    }
    const float sv = g.h_in[(size_t)hm * S + (LSTM ? H : 0) + j];
    sprev[u] = reset ? 0.0f : sv;
  }

  // GRU: r, z, n_x, n_h.  LSTM: i, f, g, o.
  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

  // PH: 0 = x chunk, 1 = h chunk, 2 = by the chunk index (the LSTM's chunks are all alike)
  auto compute = [&](int c, auto phase) {
    constexpr int PH = decltype(phase)::value;
    const int buf = c & 1;
    const float* Ab = As + (buf * BM + wm * 32 + li) * kP + 4 * lh;
    const float* Bb = Bs + (buf * NG * kBJ + li) * kP + 4 * lh;
    const bool xphase = PH == 2 ? c < nx_chunks : PH == 0;
#pragma unroll
    for (int gi = 0; gi < GPW; ++gi) {
      const int kg = (gi * WK + wk) * 8;
      const f32x4 af = *(const f32x4*)(Ab + kg);
      f32x4 bf[NG];
#pragma unroll
      for (int q = 0; q < NG; ++q) bf[q] = *(const f32x4*)(Bb + q * kBJ * kP + kg);
      if (LSTM) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int q = 0; q < NG; ++q)
            acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[q][t], acc[q], 0, 0, 0);
      } else if (xphase) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[0][t], acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[1][t], acc[1], 0, 0, 0);
          acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[2][t], acc[2], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[0][t], acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[1][t], acc[1], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[2][t], acc[3], 0, 0, 0);
        }
      }
    }
  };
  // One K group per wave and chunk (32-row blocks): the fragments of chunk c+1 are read right
  // after the barrier that publishes them, before the MFMAs of chunk c, in two register
  // slots (slot = chunk parity), so that no MFMA waits for an LDS read issued just before it.
  constexpr bool FRAG_AHEAD = GPW == 1;
  f32x4 faf[2], fbf[2][NG];
  auto rd = [&](int c, auto slotc) {
    constexpr int SL = decltype(slotc)::value;
    const int buf = c & 1, kg = wk * 8;
    faf[SL] = *(const f32x4*)(As + (buf * BM + wm * 32 + li) * kP + 4 * lh + kg);
#pragma unroll
    for (int q = 0; q < NG; ++q)
      fbf[SL][q] = *(const f32x4*)(Bs + (buf * NG * kBJ + q * kBJ + li) * kP + 4 * lh + kg);
  };
  auto mm = [&](int c, auto phase, auto slotc) {
    constexpr int PH = decltype(phase)::value, SL = decltype(slotc)::value;
    const bool xphase = PH == 2 ? c < nx_chunks : PH == 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (LSTM) {
#pragma unroll
        for (int q = 0; q < NG; ++q)
          acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(faf[SL][t], fbf[SL][q][t], acc[q], 0, 0, 0);
      } else {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(faf[SL][t], fbf[SL][0][t], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(faf[SL][t], fbf[SL][1][t], acc[1], 0, 0, 0);
        if (xphase)
          acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(faf[SL][t], fbf[SL][2][t], acc[2], 0, 0, 0);
        else
          acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(faf[SL][t], fbf[SL][2][t], acc[3], 0, 0, 0);
      }
    }
  };
  using I2 = std::integral_constant<int, 2>;
  auto step = [&](auto set, int c, auto phase, auto loadc, auto storec) {
    constexpr int SET = decltype(set)::value;
    using Other = std::integral_constant<int, SET ^ 1>;
    if (decltype(loadc)::value) gload(set, c + 2);
    if constexpr (FRAG_AHEAD) {
      if (decltype(storec)::value) sstore(Other{}, (c + 1) & 1);
      __syncthreads();
      if (decltype(storec)::value) rd(c + 1, Other{});
      mm(c, phase, set);
    } else {
      compute(c, phase);
      if (decltype(storec)::value) sstore(Other{}, (c + 1) & 1);
      __syncthreads();
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using Yes = std::true_type;
  using No = std::false_type;
  gload(I0{}, 0);
  sstore(I0{}, 0);
  if (nchunks > 1) gload(I1{}, 1);
  __syncthreads();
  if (FRAG_AHEAD) rd(0, I0{});
  if (LSTM) {
    // Steady state without a condition around the loads (with one, the compiler waits for
    // every outstanding load before each LDS store, and nothing stays in flight across a
    // chunk); the last chunks are peeled off.  Measured: 53 -> 49 us at B = 1024, H = 512.
    int c = 0;
    for (; c + 3 < nchunks; c += 2) {
      step(I0{}, c, I2{}, Yes{}, Yes{});
      step(I1{}, c + 1, I2{}, Yes{}, Yes{});
    }
    if (c + 3 == nchunks) {
      step(I0{}, c, I2{}, Yes{}, Yes{});
      step(I1{}, c + 1, I2{}, No{}, Yes{});
      step(I0{}, c + 2, I2{}, No{}, No{});
    } else if (c + 2 == nchunks) {
      step(I0{}, c, I2{}, No{}, Yes{});
      step(I1{}, c + 1, I2{}, No{}, No{});
    } else {
      step(I0{}, c, I2{}, No{}, No{});
    }
  } else if (PAIRS) {
    // GRU, x chunks and h chunks in pairs: one plain loop per accumulator set, the loads
    // running on across the change of phase, the last pair without loads.
    int c = 0;
    for (; c < nx_chunks; c += 2) {
      step(I0{}, c, I0{}, Yes{}, Yes{});
      step(I1{}, c + 1, I0{}, Yes{}, Yes{});
    }
    for (; c + 2 < nchunks; c += 2) {
      step(I0{}, c, I1{}, Yes{}, Yes{});
      step(I1{}, c + 1, I1{}, Yes{}, Yes{});
    }
    step(I0{}, c, I1{}, No{}, Yes{});
    step(I1{}, c + 1, I1{}, No{}, No{});
  } else {
    // GRU, any chunk counts: conditions around the loads and the accumulator set chosen
    // per chunk (peeling this form costs so many accumulator registers that it runs slower).
    for (int c = 0; c < nchunks; c += 2) {
      if (c + 2 < nchunks) gload(I0{}, c + 2);
      if (!FRAG_AHEAD) compute(c, I2{});
      if (c + 1 < nchunks) sstore(I1{}, (c + 1) & 1);
      __syncthreads();
      if (FRAG_AHEAD) {
        if (c + 1 < nchunks) rd(c + 1, I1{});
        mm(c, I2{}, I0{});
      }
      if (c + 1 < nchunks) {
        if (c + 3 < nchunks) gload(I1{}, c + 3);
        if (!FRAG_AHEAD) compute(c + 1, I2{});
        if (c + 2 < nchunks) sstore(I0{}, c & 1);
        __syncthreads();
        if (FRAG_AHEAD) {
          if (c + 2 < nchunks) rd(c + 2, I0{});
          mm(c + 1, I2{}, I1{});
        }
      }
    }
  }

  // Partial tiles of every wave -> LDS (the tile buffers are no longer read), two of the four
  // tiles at a time so that the exchange fits into the operand tiles' 36 KB and four
  // workgroups share a CU.  Wave wk then owns tile rows v in [wk*VPW, (wk+1)*VPW) and sums
  // the K split in the order 0, 1, ...
  float* red = smem;
  float sums[VPW][4];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (half) __syncthreads();  // the first pair has been read
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        red[((wave * 2 + tt) * 16 + v) * 64 + lane] = acc[2 * half + tt][v];
    __syncthreads();
#pragma unroll
    for (int u = 0; u < VPW; ++u) {
      const int v = wk * VPW + u;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        float a = 0.0f;
#pragma unroll
        for (int k = 0; k < WK; ++k) a += red[(((wm + WM * k) * 2 + tt) * 16 + v) * 64 + lane];
        sums[u][2 * half + tt] = a;
      }
    }
  }

  // the gates.  Only the last row block can hold rows past the end: the row check (a branch
  // per output) is compiled in for that block alone.
  auto finish = [&](auto checked) {
    constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
    for (int u = 0; u < VPW; ++u) {
      const int v = wk * VPW + u;
      const float* s = sums[u];
      const int m = m0 + wm * 32 + (v & 3) + 4 * lh + 8 * (v >> 2);
      if (!CHECK || m < B) {
        if (LSTM) {
          const float cprev = sprev[u];
          const float ig = sigmoid_acc(s[0] + bias[0]);
          const float fg = sigmoid_acc(s[1] + bias[1]);
          const float gg = tanh_acc(s[2] + bias[2]);
          const float og = sigmoid_acc(s[3] + bias[3]);
          const float cn = fg * cprev + ig * gg;
          g.h_out[(size_t)m * S + H + j] = cn;
          g.h_out[(size_t)m * S + j] = og * tanh_acc(cn);
        } else {
          const float hprev = sprev[u];
          const float r = sigmoid_acc(s[0] + bias[0]);
          const float z = sigmoid_acc(s[1] + bias[1]);
          const float n = tanh_acc(s[2] + bias[2] + r * (s[3] + bias[3]));
          g.h_out[(size_t)m * S + j] = (1.0f - z) * n + z * hprev;
        }
      }
    }
  };
  if (m0 + BM <= B)
    finish(std::false_type{});
  else
    finish(std::true_type{});
}

}  // namespace

// Every piece of the input and the state width must be whole 32-wide K chunks.
bool rnn_mfma_supported(int I1, int I2, int H) {
  return (I1 % kBK) == 0 && (I2 % kBK) == 0 && (H % kBK) == 0 && I1 > 0;
}

// Row-block size: 64 rows per workgroup when that still gives every CU several
// workgroups, else 32.  Callers fix the choice once, from the largest batch.
int rnn_mfma_pick_bm(int max_batch, int H) {
  long long wgs64 = (long long)((max_batch + 63) / 64) * (H / kBJ);
  return wgs64 >= 1024 ? 64 : 32;
}

hipError_t launch_rnn_mfma(int lstm, int B, int I1, int I2, int H, const float* x1, const float* x2,
                           const float* h_in, const uint8_t* done, const float* w_ih,
                           const float* w_hh, const float* b_ih, const float* b_hh, float* h_out,
                           int bm, int plain_loops, const int32_t* ids, int n_env, hipStream_t st) {
  if (B == 0) return hipSuccess;
  RnnArgs g;
  g.x1 = x1; g.x2 = x2; g.h_in = h_in; g.done = done;
  g.w_ih = w_ih; g.w_hh = w_hh; g.b_ih = b_ih; g.b_hh = b_hh; g.h_out = h_out;
  g.B = B; g.I1 = I1; g.I2 = x2 ? I2 : 0; g.H = H; g.ids = ids; g.n_env = n_env;
  const bool pairs = plain_loops && ((g.I1 + g.I2) % 64) == 0 && (H % 64) == 0;
  if (bm == 64) {
    dim3 grid((B + 63) / 64, H / kBJ);
    if (lstm)
      rnn_mfma_kernel<64, true, false><<<grid, 256, 0, st>>>(g);
    else
      if (pairs) rnn_mfma_kernel<64, false, true><<<grid, 256, 0, st>>>(g); else rnn_mfma_kernel<64, false, false><<<grid, 256, 0, st>>>(g);
  } else {
    dim3 grid((B + 31) / 32, H / kBJ);
    if (lstm)
      rnn_mfma_kernel<32, true, false><<<grid, 256, 0, st>>>(g);
    else
      if (pairs) rnn_mfma_kernel<32, false, true><<<grid, 256, 0, st>>>(g); else rnn_mfma_kernel<32, false, false><<<grid, 256, 0, st>>>(g);
  }
  return hipGetLastError();
}

}  // namespace sf

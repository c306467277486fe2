// Implicit-GEMM convolution and fully connected layer on the fp32 MFMA
// (paper, App. "Model architectures": conv layers 2..n and the FC layer).
//
//   out[m][n] = act(bias[n] + sum_k A[m][k] * Wt[n][k])
//
// A is never materialised: row m = (frame b, output pixel oy, ox) of a channels-last
// activation [B][H][W][Cin]; with K ordered (filter row p, filter column q, channel c)
// the K axis of a row is `ksize` contiguous segments of ksize*Cin floats, one per
// filter row (no padding).  The FC layer is the case H = W = ksize = 1.  Wt is
// [N][K] with K contiguous in the same order.
//
// Tiling: a workgroup of four wavefronts owns a BM x BN output tile, K is walked in
// chunks of 32 or 64 staged through LDS (double buffered, one barrier per chunk, global
// loads two chunks ahead of the MFMAs).  LDS rows have a pitch of BK + 4 floats so that
// both the 16-byte tile stores and the 16-byte fragment loads are bank-conflict free.
// v_mfma_f32_32x32x2_f32 takes its K index from the lane half
// h = lane/32; a lane loads four consecutive k (one ds_read_b128) at 8g + 4h, and
// instruction t of the group's four uses element t, for both operands alike.
// The four wavefronts are arranged WM x WN x WK: WK > 1 splits the K groups of
// every chunk between waves (for GEMMs with few output tiles) and the partial
// tiles are summed through LDS in a fixed order.
#include <stdlib.h>

#include <mutex>

#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;  // smallest K chunk: shapes must be multiples of it

struct GemmArgs {
  const float* A;
  const float* Wt;
  const float* bias;
  float* out;
  int M, N, K;
  // row gather
  int rows_per_img, Wo, stride, Wpix, Cin;
  long long img_elems;
  int seg_len, seg_stride;
  int relu;
};

// TAG only gives each layer of a network its own kernel symbol, so that a profiler's
// per-kernel statistics do not merge layers that share a tile configuration.
// PIPE: LDS fragment reads one K group ahead of their MFMAs (see below); it pays in grids of
// one round (FC, conv3 at B = 1024: -4 %) and costs registers and time in grids of several
// rounds (conv2: +1..5 %), so the launcher picks.
template <int BM, int BN, int BK, int WM, int WN, int WK, int TAG, bool PIPE>
__global__ __launch_bounds__(64 * WM * WN * WK) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int NT = 64 * WM * WN * WK;      // threads: one to four wavefronts
  constexpr int P = BK + 4;                  // LDS row pitch in floats
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  constexpr int TPR = BK / 4;                // threads (16-byte loads) per tile row
  constexpr int RPP = NT / TPR;              // tile rows covered by one pass of the workgroup
  constexpr int RA = BM / RPP, RB = BN / RPP;
  constexpr int NG = BK / 8;                 // K groups per chunk
  constexpr int GPW = NG / WK;               // K groups per wave per chunk
  static_assert(RA >= 1 && RB >= 1 && GPW >= 1, "tile too small for this BK");
  static_assert(GPW == 1 || GPW % 2 == 0, "fragment slots alternate with the running K group index");
  extern __shared__ float smem[];
  float* As = smem;                 // [2][BM][P]
  float* Bs = smem + 2 * BM * P;    // [2][BN][P]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = (wave / WM) % WN, wk = wave / (WM * WN);
  const int li = lane & 31, lh = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Give
  // every XCD one contiguous run of tiles (N tiles of an M tile adjacent, then the
  // next M tile), so that the rows shared by overlapping filter windows and by the
  // N tiles are re-read from that XCD's L2 instead of from memory.
  const int n_ntiles = g.N / BN;
  const int n_tiles = ((g.M + BM - 1) / BM) * n_ntiles;
  const int per_xcd = (n_tiles + 7) / 8;
  const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile_id >= n_tiles) return;
  const int m0 = (tile_id / n_ntiles) * BM, n0 = (tile_id % n_ntiles) * BN;
  const int lrow = tid / TPR, lk4 = (tid % TPR) * 4;

  const float* a_ptr[RA];
#pragma unroll
  for (int r = 0; r < RA; ++r) {
    int m = m0 + lrow + RPP * r;
    m = m < g.M ? m : g.M - 1;  // rows past the end re-read the last row; never stored
    int b = m / g.rows_per_img;
    int rem = m - b * g.rows_per_img;
    int oy = rem / g.Wo, ox = rem - oy * g.Wo;
    a_ptr[r] = g.A + (size_t)b * g.img_elems +
               ((size_t)(oy * g.stride) * g.Wpix + (size_t)ox * g.stride) * g.Cin + lk4;
  }
  const float* b_ptr[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) b_ptr[r] = g.Wt + (size_t)(n0 + lrow + RPP * r) * g.K + lk4;

  // Two register sets: global loads run two chunks ahead of the MFMAs (one chunk of
  // compute does not cover the latency of a load that misses the L2).  The load
  // cursor walks K chunk by chunk: within a row segment the A offset advances by BK,
  // at a segment's end it jumps to the next filter row.
  f32x4 ra[2][RA], rb[2][RB];
  int ld_kk = 0, ld_off = 0, ld_in_seg = 0;
  auto gload = [&](auto set) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int r = 0; r < RA; ++r) ra[S][r] = *(const f32x4*)(a_ptr[r] + ld_off);
#pragma unroll
    for (int r = 0; r < RB; ++r) rb[S][r] = *(const f32x4*)(b_ptr[r] + ld_kk);
    ld_kk += BK;
    ld_off += BK;
    ld_in_seg += BK;
    if (ld_in_seg == g.seg_len) {
      ld_in_seg = 0;
      ld_off += g.seg_stride - g.seg_len;
    }
  };
  // LDS addresses of this thread's staging stores and fragment loads, per buffer
  float* as_st = As + lrow * P + lk4;
  float* bs_st = Bs + lrow * P + lk4;
  const float* a_fr = As + (wm * TM * 32 + li) * P + 4 * lh;
  const float* b_fr = Bs + (wn * TN * 32 + li) * P + 4 * lh;
  auto sstore = [&](auto set, auto bufc) {
    constexpr int S = decltype(set)::value;
    constexpr int BUF = decltype(bufc)::value;
#pragma unroll
    for (int r = 0; r < RA; ++r) *(f32x4*)(as_st + (BUF * BM + RPP * r) * P) = ra[S][r];
#pragma unroll
    for (int r = 0; r < RB; ++r) *(f32x4*)(bs_st + (BUF * BN + RPP * r) * P) = rb[S][r];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // The bias is fetched before the K loop: after it, the load's latency would sit between
  // the last MFMA and the stores of every tile.
  float bj[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bj[j] = g.bias[n0 + (wn * TN + j) * 32 + li];

  const int nchunks = g.K / BK;
  // Fragments are read one K group ahead of their MFMAs, in two register slots (slot = parity
  // of the running group index), also across the barrier: the first group of chunk c+1 is
  // read right after the barrier that publishes it, before the MFMAs of chunk c's last group,
  // so no MFMA waits for an LDS read issued just before it.
  f32x4 af[2][TM], bf[2][TN];
  auto rd = [&](auto bufc, auto groupc, auto slotc) {
    constexpr int BUF = decltype(bufc)::value, GI = decltype(groupc)::value, SL = decltype(slotc)::value;
    const int kg = (GI * WK + wk) * 8;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[SL][i] = *(const f32x4*)(a_fr + (BUF * BM + i * 32) * P + kg);
#pragma unroll
    for (int j = 0; j < TN; ++j) bf[SL][j] = *(const f32x4*)(b_fr + (BUF * BN + j * 32) * P + kg);
  };
  auto mm = [&](auto slotc) {
    constexpr int SL = decltype(slotc)::value;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[SL][i][t], bf[SL][j][t], acc[i][j], 0, 0, 0);
  };
  // iteration c (parity S): start the loads of chunk c+2 into register set S, run the
  // MFMAs of chunk c from LDS buffer S, then move chunk c+1 (set S^1, loaded one
  // iteration ago) into LDS buffer S^1; one barrier per chunk.
  auto step = [&](auto set, auto loadc, auto storec) {
    constexpr int S = decltype(set)::value;
    using Other = std::integral_constant<int, S ^ 1>;
    if (decltype(loadc)::value) gload(set);
    if constexpr (PIPE) {
      // groups 0 .. GPW-2: read the next group, multiply this one
      auto groups = [&](auto self, auto gic) -> void {
        constexpr int GI = decltype(gic)::value;
        if constexpr (GI + 1 < GPW) {
          rd(set, std::integral_constant<int, GI + 1>{}, std::integral_constant<int, (S * GPW + GI + 1) & 1>{});
          mm(std::integral_constant<int, (S * GPW + GI) & 1>{});
          self(self, std::integral_constant<int, GI + 1>{});
        }
      };
      groups(groups, std::integral_constant<int, 0>{});
      if (decltype(storec)::value) sstore(Other{}, Other{});
      __syncthreads();
      if (decltype(storec)::value)  // there is a next chunk: its first group
        rd(Other{}, std::integral_constant<int, 0>{}, std::integral_constant<int, ((S ^ 1) * GPW) & 1>{});
      mm(std::integral_constant<int, (S * GPW + GPW - 1) & 1>{});
    } else {
      // every group read right before its MFMAs (slot 0 only)
      auto groups = [&](auto self, auto gic) -> void {
        constexpr int GI = decltype(gic)::value;
        if constexpr (GI < GPW) {
          rd(set, gic, std::integral_constant<int, 0>{});
          mm(std::integral_constant<int, 0>{});
          self(self, std::integral_constant<int, GI + 1>{});
        }
      };
      groups(groups, std::integral_constant<int, 0>{});
      if (decltype(storec)::value) sstore(Other{}, Other{});
      __syncthreads();
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using Yes = std::true_type;
  using No = std::false_type;
  gload(I0{});
  sstore(I0{}, I0{});
  if (nchunks > 1) gload(I1{});
  __syncthreads();
  if (PIPE) rd(I0{}, I0{}, I0{});
  // Steady state without conditions around the loads: a load that is issued on one path only
  // makes the compiler wait for every outstanding load before each LDS store (it must cover
  // the path without the new loads), which takes the prefetch distance from two chunks to
  // none.  The last two chunks are peeled off instead.
  int c = 0;
  for (; c + 3 < nchunks; c += 2) {
    step(I0{}, Yes{}, Yes{});
    step(I1{}, Yes{}, Yes{});
  }
  // here 1, 2 or 3 chunks remain: c + 1 <= nchunks <= c + 3
  if (c + 3 == nchunks) {
    step(I0{}, Yes{}, Yes{});
    step(I1{}, No{}, Yes{});
    step(I0{}, No{}, No{});
  } else if (c + 2 == nchunks) {
    step(I0{}, No{}, Yes{});
    step(I1{}, No{}, No{});
  } else {
    step(I0{}, No{}, No{});
  }

  // sum the K-split partial tiles in a fixed order (wk = 1, 2, 3 into wk = 0)
  if (WK > 1) {
    float* red = smem;  // [WM*WN][TM*TN][16][64] floats, reused per source wave
    for (int src = 1; src < WK; ++src) {
      if (wk == src) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              red[(((wm + WM * wn) * TM * TN + i * TN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
      }
      __syncthreads();
      if (wk == 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              acc[i][j][v] += red[(((wm + WM * wn) * TM * TN + i * TN + j) * 16 + v) * 64 + lane];
      }
      __syncthreads();
    }
    if (wk != 0) return;
  }

  // epilogue: D[i][j] of a 32x32 tile: j = lane%32, i = (v%4) + 4*(lane/32) + 8*(v/4).
  // A per-lane predicate puts a branch around every store; only the last row tile can hold
  // rows past the end, so the choice is made once per workgroup.
  auto write_tile = [&](auto checked) {
    constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + (wn * TN + j) * 32 + li;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + (wm * TM + i) * 32 + (v & 3) + 4 * lh + 8 * (v >> 2);
          float r = acc[i][j][v] + bj[j];
          if (g.relu) r = fmaxf(r, 0.0f);
          if (!CHECK || m < g.M) g.out[(size_t)m * g.N + col] = r;
        }
    }
  };
  if (m0 + BM <= g.M)
    write_tile(std::false_type{});
  else
    write_tile(std::true_type{});
}

template <int BM, int BN, int BK, int WM, int WN, int WK, int TAG, bool PIPE>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t st) {
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  if (g.K % BK != 0 || g.seg_len % BK != 0) return hipErrorInvalidValue;
  size_t lds = sizeof(float) * 2 * (BM + BN) * (BK + 4);
  size_t red = WK > 1 ? sizeof(float) * WM * WN * TM * TN * 16 * 64 : 0;
  if (red > lds) lds = red;
  auto kern = gemm_mfma_kernel<BM, BN, BK, WM, WN, WK, TAG, PIPE>;
  static std::once_flag attr_once;  // per instantiation
  static hipError_t attr_status = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_status = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)lds);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int n_tiles = ((g.M + BM - 1) / BM) * (g.N / BN);
  const int per_xcd = (n_tiles + 7) / 8;
  kern<<<per_xcd * 8, 64 * WM * WN * WK, lds, st>>>(g);
  return hipGetLastError();
}

template <int TAG>
hipError_t launch_tile(const GemmArgs& g, int tile, hipStream_t st) {
  const bool n64 = (g.N % 64) == 0;
  switch (tile) {
    case 1: return n64 ? launch_cfg<128, 64, 32, 4, 1, 1, TAG, false>(g, st) : hipErrorInvalidValue;
    case 2: return n64 ? launch_cfg<64, 64, 32, 2, 2, 1, TAG, true>(g, st) : hipErrorInvalidValue;
    case 3: {
      // one round of workgroups (5 per CU): fragment reads pipelined; results are the same bits
      const long long n_tiles = (long long)((g.M + 63) / 64) * (g.N / 32);
      return n_tiles <= 1280 ? launch_cfg<64, 32, 32, 2, 1, 2, TAG, true>(g, st)
                             : launch_cfg<64, 32, 32, 2, 1, 2, TAG, false>(g, st);
    }
    case 4: return launch_cfg<32, 32, 32, 1, 1, 4, TAG, true>(g, st);
    case 6: return launch_cfg<64, 32, 64, 2, 1, 2, TAG, false>(g, st);
    case 7: return launch_cfg<32, 32, 64, 1, 1, 4, TAG, true>(g, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Shapes the kernel accepts: no padding, channel count and row segment multiples of
// 32 / 4, N a multiple of 32.
bool gemm_mfma_supported(int Cin, int ksize, int pad, int N) {
  return pad == 0 && (Cin % 4) == 0 && ((ksize * Cin) % kBK) == 0 && (N % 32) == 0;
}

// Tile configuration for an M x N x K problem, measured on MI355X.  Grids of several rounds
// of workgroups (conv2 from B = 1024, conv3 from B = 2048) run best on the 64x64 tile (each
// wave one 32x32 block over the whole K, no K-split reduction, fragment reads pipelined);
// below that the 64x32 tile with a two-way in-workgroup K split wins as long as it yields
// about a thousand workgroups, and the 32x32 tile with a four-way K split (chunks of 64
// where K allows) otherwise.  Callers fix the choice once (from the largest batch) so that
// results do not depend on the batch size of a call.
int gemm_mfma_pick_tile(long long M, int N, int K, int seg_len) {
  if ((N % 64) == 0 && ((M + 63) / 64) * (N / 64) >= 1024) return 2;
  long long wgs = ((M + 63) / 64) * (N / 32);
  if (wgs >= 1024) return 3;
  return (K % 64 == 0 && seg_len % 64 == 0) ? 7 : 4;
}

hipError_t launch_gemm_mfma(const float* A, const float* Wt, const float* bias, float* out, int B,
                            int H, int W, int Cin, int ksize, int stride, int Ho, int Wo, int N,
                            int relu, int tile_hint, int tag, hipStream_t st) {
  GemmArgs g;
  g.A = A; g.Wt = Wt; g.bias = bias; g.out = out;
  g.M = B * Ho * Wo; g.N = N; g.K = ksize * ksize * Cin;
  g.rows_per_img = Ho * Wo; g.Wo = Wo; g.stride = stride; g.Wpix = W; g.Cin = Cin;
  g.img_elems = (long long)H * W * Cin;
  g.seg_len = ksize * Cin; g.seg_stride = W * Cin;
  g.relu = relu;
  if (g.M == 0) return hipSuccess;
  const int tile = tile_hint > 0 ? tile_hint : gemm_mfma_pick_tile(g.M, N, g.K, g.seg_len);
  switch (tag & 3) {
    case 0: return launch_tile<0>(g, tile, st);
    case 1: return launch_tile<1>(g, tile, st);
    case 2: return launch_tile<2>(g, tile, st);
    default: return launch_tile<3>(g, tile, st);
  }
}

}  // namespace sf

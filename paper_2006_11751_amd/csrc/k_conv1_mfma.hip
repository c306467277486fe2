// First convolution of the plain encoder as an implicit GEMM on the fp32 MFMA
// (paper, App. "Model architectures": the convolutional encoder reads the pixel
// observation).  Specialised for an 8x8 filter with stride 4, no padding, 32 output
// channels, reading planar byte frames directly: the frame load, the byte->float
// conversion and the normalisation never touch memory as floats.
//
// GEMM view per frame: M = Ho*Wo output pixels, N = 32 channels, K = Cin*8*8.
// One wavefront owns a run of (frame, output row, 32-pixel column chunk) items.
// The whole 192x32 filter bank lives in the wave's registers for the duration
// (the normalisation x = (byte - sub) * mul is folded into it and into the bias
// when the weights are packed), so the only operand traffic per item is one dword
// (4 horizontally adjacent bytes) per lane per (channel, filter row).
// With sub != 0 the A operand is byte - c, c = sub rounded to a byte value, and the
// bias absorbs the rest: the fp32 sums then stay of the size of the normalised
// pixels' terms instead of cancelling against a large bias.
//
// v_mfma_f32_32x32x2_f32: lane l supplies A[i = l%32][k = l/32] and
// B[k = l/32][j = l%32]; the K index inside one instruction is therefore the lane
// half h = l/32.  K is ordered so that for a fixed (channel c, filter row p) the
// lane half h holds filter columns q = 4h..4h+3, and instruction t of the four
// consumes column q = 4h + t: exactly byte t of the dword the lane loaded.
#include <math.h>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kCout = 32;
constexpr int kK = 8;       // filter size
constexpr int kS = 4;       // stride
constexpr int kWaves = 4;   // per workgroup

template <int CIN, bool CENTER>
__global__ __launch_bounds__(64 * kWaves, 2) void conv1_u8_mfma_kernel(
    const uint8_t* __restrict__ obs, const float* __restrict__ wpk, const float* __restrict__ bias,
    float* __restrict__ out, float* __restrict__ trash, int H, int W, int Ho, int Wo,
    int n_xchunks, long long n_items, int n_waves_total, float center) {
  constexpr int NG = CIN * kK;  // (channel, filter row) groups; 4 MFMAs each
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int n = lane & 31;   // output channel (B column) / pixel within chunk (A row)
  const int h = lane >> 5;   // lane half = K slot

  // filter bank: wreg[g][t] = W'[n][c][p][q = 4h + t], packed as [g][t][lane]
  float wreg[NG][4];
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int t = 0; t < 4; ++t) wreg[g][t] = wpk[(g * 4 + t) * 64 + lane];
  const float bias_n = bias[n];

  // contiguous run of items for this wave
  const long long per = n_items / n_waves_total, rem = n_items % n_waves_total;
  long long it = wave * per + (wave < rem ? wave : rem);
  const long long it_end = it + per + (wave < rem ? 1 : 0);
  if (it >= it_end) return;

  const size_t frame_bytes = (size_t)CIN * H * W;
  const int items_per_frame = Ho * n_xchunks;

  auto item_src = [&](long long item, int& oy, int& xc) -> const uint8_t* {
    long long b = item / items_per_frame;
    int r = (int)(item - b * items_per_frame);
    oy = r / n_xchunks;
    xc = r - oy * n_xchunks;
    int ox = xc * 32 + n;
    if (ox > Wo - 1) ox = Wo - 1;  // lanes past the row end re-read the last pixel; never stored
    return obs + (size_t)b * frame_bytes + (size_t)(oy * kS) * W + ox * kS + h * 4;
  };

  uint32_t cur[NG], nxt[NG];
  int oy, xc;
  {
    const uint8_t* src = item_src(it, oy, xc);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int c = g / kK, p = g % kK;
      cur[g] = *(const uint32_t*)(src + ((size_t)c * H + p) * W);
    }
  }
  for (; it < it_end; ++it) {
    int oy_n = 0, xc_n = 0;
    const bool more = it + 1 < it_end;
    if (more) {
      const uint8_t* src = item_src(it + 1, oy_n, xc_n);
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int c = g / kK, p = g % kK;
        nxt[g] = *(const uint32_t*)(src + ((size_t)c * H + p) * W);
      }
    }
    // One accumulation chain of 4*NG MFMAs.  The byte->float conversions of the next
    // pair of groups are placed ahead of the eight MFMAs of the current pair
    // (sched_group_barrier: 8 VALU, then 8 MFMA), so that the matrix pipe gets
    // uninterrupted runs: every other instruction issued between two MFMAs of a wave
    // delays the second one.
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = bias_n;
    float a_cur[8], a_nxt[8];
    auto pixel = [&](uint32_t word, int t) -> float {
      const float v = (float)((word >> (8 * t)) & 0xFFu);
      return CENTER ? v - center : v;
    };
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      a_cur[t] = pixel(cur[0], t);
      a_cur[4 + t] = pixel(cur[1], t);
    }
#pragma unroll
    for (int g = 0; g < NG; g += 2) {
      if (g + 2 < NG) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          a_nxt[t] = pixel(cur[g + 2], t);
          a_nxt[4 + t] = pixel(cur[g + 3], t);
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[t], wreg[g][t], acc, 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 4; ++t)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[4 + t], wreg[g + 1][t], acc, 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, CENTER ? 16 : 8, 0);  // VALU: the conversions
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);  // MFMA
#pragma unroll
      for (int t = 0; t < 8; ++t) a_cur[t] = a_nxt[t];
    }
    // epilogue: ReLU, channels-last store.  D[i][j]: j = n, i = (v%4) + 4h + 8(v/4).
    // Lanes past the row end loaded the last pixel's bytes, so their result rows are
    // bitwise copies of that pixel's: storing them to its address is harmless and
    // keeps the stores unconditional.
    const long long b = it / items_per_frame;
    float* dst = out + (((size_t)b * Ho + oy) * Wo) * kCout + n;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int ox = xc * 32 + (v & 3) + 4 * h + 8 * (v >> 2);
      ox = ox < Wo ? ox : Wo - 1;
      dst[ox * kCout] = fmaxf(acc[v], 0.0f);
    }
    if (more) {
#pragma unroll
      for (int g = 0; g < NG; ++g) cur[g] = nxt[g];
      oy = oy_n;
      xc = xc_n;
    }
  }
}

}  // namespace

bool conv1_mfma_supported(const ConvLayer& L) {
  return L.k == kK && L.s == kS && L.pad == 0 && L.cout == kCout && (L.W % 4) == 0 &&
         (L.cin == 3 || L.cin == 1 || L.cin == 4) && L.relu_out == 1 && !L.add_residual;
}

// Packed filter bank for the kernel above, with the normalisation folded in:
// wpk[((c*8 + p)*4 + t)*64 + lane] = mul * w[n = lane%32][c][p][q = 4*(lane/32) + t],
// bias'[n] = bias[n] - (sub - center) * mul * sum(w[n]), center = conv1_mfma_center(sub).
float conv1_mfma_center(float obs_sub) {
  if (obs_sub == 0.0f) return 0.0f;
  const float c = nearbyintf(obs_sub);
  return c < 0.0f ? 0.0f : (c > 255.0f ? 255.0f : c);
}

void conv1_mfma_pack(const float* w, const float* bias, int cin, float obs_sub, float obs_mul,
                     std::vector<float>& wpk, std::vector<float>& bpk) {
  const double shift = (double)obs_sub - (double)conv1_mfma_center(obs_sub);
  wpk.assign((size_t)cin * kK * 4 * 64, 0.0f);
  bpk.assign(kCout, 0.0f);
  for (int c = 0; c < cin; ++c)
    for (int p = 0; p < kK; ++p)
      for (int t = 0; t < 4; ++t)
        for (int lane = 0; lane < 64; ++lane) {
          int n = lane & 31, q = 4 * (lane >> 5) + t;
          wpk[((size_t)(c * kK + p) * 4 + t) * 64 + lane] =
              obs_mul * w[(((size_t)n * cin + c) * kK + p) * kK + q];
        }
  for (int n = 0; n < kCout; ++n) {
    double s = 0.0;  // over the fp32 products the kernel multiplies by
    for (int i = 0; i < cin * kK * kK; ++i) s += (double)(obs_mul * w[(size_t)n * cin * kK * kK + i]);
    bpk[n] = (float)((double)bias[n] - shift * s);
  }
}

hipError_t launch_conv1_mfma(const ConvLayer& L, int B, const uint8_t* obs, const float* wpk,
                             const float* bpk, float* out, float* trash, int waves_hint,
                             float obs_sub, hipStream_t st) {
  if (B == 0) return hipSuccess;
  const int n_xchunks = (L.Wo + 31) / 32;
  const long long n_items = (long long)B * L.Ho * n_xchunks;
  long long waves = waves_hint > 0 ? waves_hint : 2048;  // two wavefronts per SIMD on 256 CUs
  if (waves > n_items) waves = n_items;
  const int blocks = (int)((waves + kWaves - 1) / kWaves);
  const int n_waves_total = blocks * kWaves;
  const float center = conv1_mfma_center(obs_sub);
#define SF_LAUNCH_CIN(C)                                                                          \
  do {                                                                                            \
    if (center != 0.0f)                                                                           \
      conv1_u8_mfma_kernel<C, true><<<blocks, 64 * kWaves, 0, st>>>(                              \
          obs, wpk, bpk, out, trash, L.H, L.W, L.Ho, L.Wo, n_xchunks, n_items, n_waves_total, center); \
    else                                                                                          \
      conv1_u8_mfma_kernel<C, false><<<blocks, 64 * kWaves, 0, st>>>(                             \
          obs, wpk, bpk, out, trash, L.H, L.W, L.Ho, L.Wo, n_xchunks, n_items, n_waves_total, center); \
  } while (0)
  switch (L.cin) {
    case 1: SF_LAUNCH_CIN(1); break;
    case 3: SF_LAUNCH_CIN(3); break;
    case 4: SF_LAUNCH_CIN(4); break;
    default: return hipErrorInvalidValue;
  }
#undef SF_LAUNCH_CIN
  return hipGetLastError();
}

}  // namespace sf

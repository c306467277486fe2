// First convolution of the plain encoder on the int8 MFMA, exact in the pixels
// (paper, App. "Model architectures": the convolutional encoder reads the pixel
// observation).  Same shape as the fp32 kernel: 8x8 filter, stride 4, no padding,
// 32 output channels, planar byte frames.
//
// The observation is bytes, so the convolution is an integer contraction in the
// pixels.  Per output channel n the (normalisation-folded) filter W'[.][n] is
// written in three signed digits of radix 254 with one scale s_n = max_k |W'[k][n]| / 127,
//   W'[k][n] ~= s_n * (d1[k][n] + d2[k][n] / 254 + d3[k][n] / 254^2),   |d| <= 127
// (each remainder lies in [-1/2, 1/2], so 254 is the largest radix whose next digit still
// fits a signed byte).  This is fixed point, not floating point: every tap of a channel
// carries the same ABSOLUTE error, at most s_n / (2 * 254^2) = 2^-24 of the channel's
// largest tap, whatever the tap's own size.  A tap half as large as the largest is held as
// well as fp32 holds it; a tap 1000 times smaller keeps 14 bits.  Whether that is good
// enough is decided per filter bank when it is packed (conv1_i8_pack below); a bank that
// fails the test runs on the fp32 MFMA kernel instead.  With x_s = byte - 128 (one XOR
// per four pixels) the three sums S_i = sum_k x_s[k] * d_i[k][n] are exact int32 values
// from v_mfma_i32_32x32x32_i8, which runs at 32x the rate of the fp32 MFMA and takes the
// loaded frame words as operands without any conversion:
//   out = relu(s_n * (S1 + S2/254 + S3/254^2) + b''_n),
//   b''_n = b_n - sub*mul*sum_k W[k][n] + 128 * sum_k W'[k][n]   (exact W').
//
// v_mfma_i32_32x32x32_i8: lane l supplies 16 bytes A[i = l%32][k = 16*(l/32) + e] and
// B[k = 16*(l/32) + e][j = l%32].  One instruction covers four (channel, filter row)
// groups of 8 filter columns: lane half h holds groups 4s+2h and 4s+2h+1, i.e. two
// 8-byte runs of the frame.  A wave walks a contiguous run of (frame, output row, x chunk)
// items, three register sets of frame bytes in rotation (loads two items ahead).
#include <math.h>
#include <string.h>

#include <algorithm>

#include "sf_internal.h"

namespace sf {

namespace {

typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kCout = 32;
constexpr int kK = 8;
constexpr int kS = 4;
constexpr int kWaves = 4;

struct __attribute__((packed, aligned(4))) U2 {
  uint32_t x, y;
};

constexpr float kInvRadix = 1.0f / 254.0f;
constexpr float kInvRadix2 = 1.0f / 64516.0f;

// ND: digit planes used (2 or 3; the packed bank always holds three).
template <int CIN, bool OUT_BF16, int ND>
__global__ __launch_bounds__(64 * kWaves, (CIN <= 3 ? 2 : 1)) void conv1_u8_i8_kernel(
    const uint8_t* __restrict__ obs, const int* __restrict__ wpk, const float* __restrict__ scale,
    const float* __restrict__ bias, void* __restrict__ out_v, int H, int W, int Ho, int Wo,
    int n_xchunks, long long n_items, int n_waves_total) {
  constexpr int NSTEP = CIN * kK / 4;  // MFMA K steps (32 bytes each)
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int n = lane & 31;
  const int h = lane >> 5;

  // digit planes of the filter bank: wd[s][digit] = 16 bytes of this lane's B operand
  i32x4 wd[NSTEP][ND];
#pragma unroll
  for (int s = 0; s < NSTEP; ++s)
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
      for (int w = 0; w < 4; ++w) wd[s][d][w] = wpk[((s * 3 + d) * 4 + w) * 64 + lane];
  const float s_n = scale[n], b_n = bias[n];

  // Items are dealt in contiguous runs, so everything that names an item (frame, output row,
  // x chunk, the two base addresses) is the same for the 64 lanes and lives in scalar
  // registers; it moves from item to item by carries, without divisions.  The vector ALU is
  // what bounds this kernel once the addresses are out of it.
  const long long per = n_items / n_waves_total, rem = n_items % n_waves_total;
  const long long first = wave * per + (wave < rem ? wave : rem);
  int count = (int)(per + (wave < rem ? 1 : 0));
  count = __builtin_amdgcn_readfirstlane(count);
  if (count <= 0) return;

  const int items_per_frame = Ho * n_xchunks;
  const long long frame0 = first / items_per_frame;
  const int r0 = (int)(first - frame0 * items_per_frame);
  int oy = __builtin_amdgcn_readfirstlane(r0 / n_xchunks);
  int xc = __builtin_amdgcn_readfirstlane(r0 % n_xchunks);
  const size_t frame_bytes = (size_t)CIN * H * W;
  constexpr int ELT = OUT_BF16 ? 2 : 4;
  const size_t out_row_bytes = (size_t)Wo * kCout * ELT;
  size_t in_off = (size_t)frame0 * frame_bytes + (size_t)(oy * kS) * W;      // frame, first input row
  size_t out_off = ((size_t)frame0 * Ho + oy) * out_row_bytes;               // frame, output row
  auto uniform = [](size_t v) -> size_t {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((size_t)hi << 32) | lo;
  };
  in_off = uniform(in_off);
  out_off = uniform(out_off);

  // per-lane parts: the (channel, filter row) group offsets of the 2*NSTEP loads, and the
  // output offset of tile row 4h, channel n
  uint32_t goff[NSTEP][2];
#pragma unroll
  for (int s = 0; s < NSTEP; ++s)
#pragma unroll
    for (int pp = 0; pp < 2; ++pp) {
      const int g = 4 * s + 2 * h + pp;  // (channel, filter row) group
      goff[s][pp] = (uint32_t)(((g / kK) * H + (g % kK)) * W);
    }
  // byte offset of tile row (v%4) + 8(v/4) + 4h, channel n, within the item's 32 output
  // pixels; rows past the end of the image row point at its last pixel
  uint32_t voff[16];
  auto set_store_offsets = [&](int xchunk) {
    const int nvalid = Wo - xchunk * 32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int i = (v & 3) + 8 * (v >> 2) + 4 * h;
      i = i < nvalid ? i : nvalid - 1;
      voff[v] = (uint32_t)((i * kCout + n) * ELT);
    }
  };
  set_store_offsets(xc);

  // lanes past the row end repeat the last pixel (and store nothing)
  auto lane_x = [&](int xchunk) -> uint32_t {
    int ox = xchunk * 32 + n;
    ox = ox < Wo ? ox : Wo - 1;
    return (uint32_t)(ox * kS);
  };
  auto load_item = [&](size_t ioff, uint32_t lx, U2 (&dst)[NSTEP][2]) {
    const uint8_t* base = obs + ioff;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s)
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) dst[s][pp] = *(const U2*)(base + (goff[s][pp] + lx));
  };

  // One item of compute (about 0.5 us) does not cover a load from memory: three register
  // sets, loads two items ahead of the MFMAs, roles rotating without copies.  The load
  // cursor (lx, ly, l_in) runs ahead of the compute cursor (xc, oy, out_off).
  int lx = xc, ly = oy;
  size_t l_in = in_off;
  auto advance_load = [&]() {
    if (++lx == n_xchunks) {
      lx = 0;
      l_in += (size_t)kS * W;
      if (++ly == Ho) {  // next frame: its rows follow this frame's last filter window
        ly = 0;
        l_in += frame_bytes - (size_t)Ho * kS * W;
      }
    }
  };
  int issued = 0;
  auto issue = [&](U2 (&dst)[NSTEP][2]) {
    if (issued < count) {
      load_item(l_in, lane_x(lx), dst);
      advance_load();
    }
    ++issued;
  };
  auto run_item = [&](const U2 (&cur)[NSTEP][2]) {
    i32x16 s1, s2, s3;
#pragma unroll
    for (int v = 0; v < 16; ++v) s1[v] = s2[v] = s3[v] = 0;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
      i32x4 a;  // byte - 128 on all 16 pixels of the two runs
      a[0] = (int)(cur[s][0].x ^ 0x80808080u);
      a[1] = (int)(cur[s][0].y ^ 0x80808080u);
      a[2] = (int)(cur[s][1].x ^ 0x80808080u);
      a[3] = (int)(cur[s][1].y ^ 0x80808080u);
      s1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][0], s1, 0, 0, 0);
      s2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][1], s2, 0, 0, 0);
      if constexpr (ND == 3) s3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][2], s3, 0, 0, 0);
    }
    // epilogue.  D[i][j]: j = n, i = (v%4) + 4h + 8(v/4).  S2*254 + S3 fits int32
    // (|S2|, |S3| <= 256*128*127 = 4.2e6); its float image is exact to 6e-8 relative.
    float r[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float q;
      if constexpr (ND == 3) {
        const float lo = (float)(s2[v] * 254 + s3[v]);
        q = fmaf(lo, kInvRadix2, (float)s1[v]);
      } else {
        q = fmaf((float)s2[v], kInvRadix, (float)s1[v]);
      }
      r[v] = fmaxf(fmaf(q, s_n, b_n), 0.0f);
    }
    // no predicated stores (each would become a branch): lanes past the row end write the
    // last pixel again, with the same bits
    uint8_t* obase = (uint8_t*)out_v + out_off + (size_t)(xc * 32) * (kCout * ELT);
    if (n_xchunks > 1) set_store_offsets(xc);
    if (OUT_BF16) {
      // Neighbouring lanes (channels n, n^1) swap half of their rows: the even lane keeps
      // tile rows 2k, the odd lane rows 2k+1, each as a (channel n&~1, channel n|1) pair in
      // one 32-bit word: 8 stores per item instead of 16 (a wave can have 63 memory
      // instructions outstanding, and 12 loads + 16 stores per item run into that).
      const bool odd = (n & 1) != 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float mine = odd ? r[2 * k + 1] : r[2 * k];
        const float give = odd ? r[2 * k] : r[2 * k + 1];
        const float got = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(give), 0xB1, 0xF, 0xF, true));
        const f32x2 pair = {odd ? got : mine, odd ? mine : got};
        const unsigned word = __builtin_bit_cast(unsigned, __builtin_convertvector(pair, bf16x2));
        const uint32_t off = (odd ? voff[2 * k + 1] : voff[2 * k]) - (odd ? ELT : 0);
        *(uint32_t*)(obase + off) = word;
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) *(float*)(obase + voff[v]) = r[v];
    }
    if (++xc == n_xchunks) {
      xc = 0;
      out_off += out_row_bytes;  // output rows of consecutive frames are contiguous
    }
  };

  U2 b0[NSTEP][2], b1[NSTEP][2], b2[NSTEP][2];
  issue(b0);
  issue(b1);
  for (int i = 0; i < count; i += 3) {
    issue(b2);
    run_item(b0);
    if (i + 1 < count) {
      issue(b0);
      run_item(b1);
    }
    if (i + 2 < count) {
      issue(b1);
      run_item(b2);
    }
  }
}


// The same layer with the frame resident in LDS.  The kernel above gathers its A operands
// from memory as 8-byte runs (every frame byte is fetched four times, from two filter-window
// columns and two window rows, and a wave at two per SIMD cannot cover the latency of those
// gathers).  Here a workgroup walks frames b, b + gridDim.x, ...: the whole planar byte frame
// (CIN x H x W <= 28 KB) is copied into LDS with 16-byte loads, the next frame travels into
// registers while the current one is computed, and the 8-byte runs are LDS reads.  Wave w
// takes output rows w, w + 4, ...; MFMA sequence, epilogue and stores are those of the kernel
// above (same bits).  One x chunk (Wo <= 32) and 16-byte aligned frames only.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int CIN, bool OUT_BF16, int ND>
__global__ __launch_bounds__(64 * kWaves, 2) void conv1_u8_i8_image_kernel(
    const uint8_t* __restrict__ obs, const int* __restrict__ wpk, const float* __restrict__ scale,
    const float* __restrict__ bias, void* __restrict__ out_v, int B, int H, int W, int Ho, int Wo) {
  constexpr int NSTEP = CIN * kK / 4;
  constexpr int NV = 7;  // 16-byte pieces per thread: frames up to 7 * 256 * 16 = 28672 bytes
  constexpr int NT = 64 * kWaves;
  extern __shared__ __attribute__((aligned(16))) uint8_t frame_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31;
  const int h = lane >> 5;

  i32x4 wd[NSTEP][ND];
#pragma unroll
  for (int s = 0; s < NSTEP; ++s)
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
      for (int w = 0; w < 4; ++w) wd[s][d][w] = wpk[((s * 3 + d) * 4 + w) * 64 + lane];
  const float s_n = scale[n], b_n = bias[n];

  const int frame_bytes = CIN * H * W;
  const int pieces = frame_bytes / 16;
  constexpr int ELT = OUT_BF16 ? 2 : 4;
  const size_t out_row_bytes = (size_t)Wo * kCout * ELT;

  // LDS byte offset of this lane's two runs per MFMA step at output row 0: (channel, filter
  // row) group g = 4s + 2h + pp, output pixel n (lanes past the row end repeat the last pixel)
  int ox = n < Wo ? n : Wo - 1;
  uint32_t goff[NSTEP][2];
#pragma unroll
  for (int s = 0; s < NSTEP; ++s)
#pragma unroll
    for (int pp = 0; pp < 2; ++pp) {
      const int g = 4 * s + 2 * h + pp;
      goff[s][pp] = (uint32_t)(((g / kK) * H + (g % kK)) * W + ox * kS);
    }
  // byte offset of tile row (v%4) + 8(v/4) + 4h, channel n, within the output row; rows past
  // the end point at the last pixel (stored again with the same bits)
  uint32_t voff[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    int i = (v & 3) + 8 * (v >> 2) + 4 * h;
    i = i < Wo ? i : Wo - 1;
    voff[v] = (uint32_t)((i * kCout + n) * ELT);
  }

  u32x4 fv[NV];
  auto load_frame = [&](int b) {
    const u32x4* src = (const u32x4*)(obs + (size_t)b * frame_bytes);
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int f = tid + NT * u;
      fv[u] = src[f < pieces ? f : pieces - 1];
    }
  };
  auto load_row = [&](int oy, U2 (&dst)[NSTEP][2]) {
    const uint8_t* base = frame_lds + (size_t)(oy * kS) * W;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s)
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) dst[s][pp] = *(const U2*)(base + goff[s][pp]);
  };
  i32x16 s1, s2, s3;
  auto multiply_row = [&](const U2 (&cur)[NSTEP][2]) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s1[v] = s2[v] = s3[v] = 0;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
      i32x4 a;  // byte - 128 on all 16 pixels of the two runs
      a[0] = (int)(cur[s][0].x ^ 0x80808080u);
      a[1] = (int)(cur[s][0].y ^ 0x80808080u);
      a[2] = (int)(cur[s][1].x ^ 0x80808080u);
      a[3] = (int)(cur[s][1].y ^ 0x80808080u);
      s1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][0], s1, 0, 0, 0);
      s2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][1], s2, 0, 0, 0);
      if constexpr (ND == 3) s3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][2], s3, 0, 0, 0);
    }
  };
  auto finish_row = [&](uint8_t* obase) {
    float r[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float q;
      if constexpr (ND == 3) {
        const float lo = (float)(s2[v] * 254 + s3[v]);
        q = fmaf(lo, kInvRadix2, (float)s1[v]);
      } else {
        q = fmaf((float)s2[v], kInvRadix, (float)s1[v]);
      }
      r[v] = fmaxf(fmaf(q, s_n, b_n), 0.0f);
    }
    if (OUT_BF16) {
      const bool odd = (n & 1) != 0;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float mine = odd ? r[2 * k + 1] : r[2 * k];
        const float give = odd ? r[2 * k] : r[2 * k + 1];
        const float got = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(give), 0xB1, 0xF, 0xF, true));
        const f32x2 pair = {odd ? got : mine, odd ? mine : got};
        const unsigned word = __builtin_bit_cast(unsigned, __builtin_convertvector(pair, bf16x2));
        const uint32_t off = (odd ? voff[2 * k + 1] : voff[2 * k]) - (odd ? ELT : 0);
        *(uint32_t*)(obase + off) = word;
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) *(float*)(obase + voff[v]) = r[v];
    }
  };

  int b = blockIdx.x;
  load_frame(b);
  for (; b < B; b += gridDim.x) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int f = tid + NT * u;
      *(u32x4*)(frame_lds + 16 * (size_t)(f < pieces ? f : pieces - 1)) = fv[u];
    }
    __syncthreads();
    load_frame(b + (int)gridDim.x < B ? b + (int)gridDim.x : b);  // (last round: its own again)

    uint8_t* oframe = (uint8_t*)out_v + (size_t)b * Ho * out_row_bytes;
    // one set of row bytes: the wave's next row is read behind this row's MFMAs, under its
    // epilogue (past the wave's last row: that row again, unused)
    U2 rb[NSTEP][2];
    int oy = wv;
    if (oy < Ho) load_row(oy, rb);
    for (; oy < Ho; oy += kWaves) {
      multiply_row(rb);
      load_row(oy + kWaves < Ho ? oy + kWaves : oy, rb);
      finish_row(oframe + (size_t)oy * out_row_bytes);
    }
    __syncthreads();  // every wave is done with this frame
  }
}

}  // namespace

bool conv1_i8_supported(const ConvLayer& L) {
  return L.k == kK && L.s == kS && L.pad == 0 && L.cout == kCout && (L.W % 4) == 0 &&
         (L.cin == 3 || L.cin == 1 || L.cin == 4) && L.relu_out == 1 && !L.add_residual;
}

// Digit planes, scales and bias for the kernels above, and the test that decides whether
// the fixed-point bank may stand in for floating-point weights.
// wpk[((s*3 + d)*4 + w)*64 + lane]: bytes e = 4w..4w+3 of the lane's operand for K step s
// and digit d; byte e belongs to group g = 4s + 2*(lane/32) + e/8 = (channel g/8, filter
// row g%8), filter column e%8, output channel lane%32.
//
// The test, per output channel, in fp64 on the packed digits themselves.  The kernel's
// result differs from the exact one by sum_k x_s[k] * (W'[k] - What[k]) with |x_s| <= 128, so
//   E_fix = 128 * sum_k |W'[k] - What[k]|
// bounds its error for every frame.  It is held against the error of the floating-point
// path the bank replaces, for a full-scale frame, with every tap counted at no more than
// the channel's median non-zero tap m (so that a few dominant taps cannot buy slack for the
// many small ones, whose terms are what is left of the output when the dominant taps sit on
// dark pixels):
//   fp32 bank, three planes: E_ref = sqrt(K) * 2^-24 * 255 * sum_k min(|W'[k]|, m)
//                            (random-walk estimate of K roundings of an fp32 accumulation)
//   bf16 bank, two planes:   E_ref = 2^-9 * 255 * sum_k min(|W'[k]|, m)
//                            (the rounding to bf16 that the configuration applies to the
//                            same taps)
// ratio = max over channels of E_fix / E_ref; the bank is admitted when ratio <= 1.  Gaussian
// filters give about 0.1 (three planes); a filter with one tap 1000 times the others about 45.
void conv1_i8_pack(const float* w, const float* bias, int cin, float obs_sub, float obs_mul,
                   bool bf16_weights, std::vector<int>& wpk, std::vector<float>& scale,
                   std::vector<float>& bpk, Conv1I8Info* info) {
  const int K = cin * kK * kK;
  const int nstep = cin * kK / 4;
  wpk.assign((size_t)nstep * 3 * 4 * 64, 0);
  scale.assign(kCout, 1.0f);
  bpk.assign(kCout, 0.0f);
  std::vector<signed char> dig((size_t)kCout * K * 3);
  std::vector<double> wm(K), mag(K);
  double worst2 = 0.0, worst3 = 0.0;
  // a bf16 configuration defines its parameters as the nearest bf16 values (ties to even)
  auto param = [&](float v) -> double {
    if (bf16_weights) {
      uint32_t u;
      memcpy(&u, &v, 4);
      if ((u & 0x7F800000u) != 0x7F800000u) u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
      memcpy(&v, &u, 4);
    }
    return (double)v;
  };
  auto tap = [&](int n, int i) -> double { return param(w[(size_t)n * K + i]); };
  auto clamp_digit = [](double d) { return d > 127 ? 127.0 : (d < -127 ? -127.0 : d); };
  for (int n = 0; n < kCout; ++n) {
    double mx = 0.0, sum_w = 0.0, sum_wm = 0.0;
    for (int i = 0; i < K; ++i) {
      const double wi = tap(n, i);
      wm[i] = (double)obs_mul * wi;
      mx = fmax(mx, fabs(wm[i]));
      sum_w += wi;
      sum_wm += wm[i];
    }
    const float sf = mx > 0.0 ? (float)(mx / 127.0) : 1.0f;  // the kernel multiplies by this fp32 value
    const double s = (double)sf;
    double res2 = 0.0, res3 = 0.0;
    int nz = 0;
    for (int i = 0; i < K; ++i) {
      const double q = wm[i] / s;
      const double d1 = clamp_digit(nearbyint(q));
      const double r = (q - d1) * 254.0;
      const double d2 = clamp_digit(nearbyint(r));
      const double d3 = clamp_digit(nearbyint((r - d2) * 254.0));
      dig[((size_t)n * K + i) * 3 + 0] = (signed char)d1;
      dig[((size_t)n * K + i) * 3 + 1] = (signed char)d2;
      dig[((size_t)n * K + i) * 3 + 2] = (signed char)d3;
      res2 += fabs(wm[i] - s * (d1 + d2 / 254.0));
      res3 += fabs(wm[i] - s * (d1 + d2 / 254.0 + d3 / 64516.0));
      if (wm[i] != 0.0) mag[nz++] = fabs(wm[i]);
    }
    if (nz > 0) {
      std::nth_element(mag.begin(), mag.begin() + (nz - 1) / 2, mag.begin() + nz);
      const double m = mag[(nz - 1) / 2];
      double l1 = 0.0;
      for (int i = 0; i < K; ++i) l1 += fmin(fabs(wm[i]), m);
      const double ref3 = sqrt((double)K) * 0x1.0p-24 * 255.0 * l1;
      const double ref2 = 0x1.0p-9 * 255.0 * l1;
      worst3 = fmax(worst3, 128.0 * res3 / ref3);
      worst2 = fmax(worst2, 128.0 * res2 / ref2);
    }
    scale[n] = sf;
    bpk[n] = (float)(param(bias[n]) - (double)obs_sub * (double)obs_mul * sum_w + 128.0 * sum_wm);
  }
  if (info) {
    info->ratio2 = worst2;
    info->ratio3 = worst3;
  }
  for (int s = 0; s < nstep; ++s)
    for (int d = 0; d < 3; ++d)
      for (int wq = 0; wq < 4; ++wq)
        for (int lane = 0; lane < 64; ++lane) {
          const int n = lane & 31, hh = lane >> 5;
          uint32_t word = 0;
          for (int e4 = 0; e4 < 4; ++e4) {
            const int e = 4 * wq + e4;
            const int g = 4 * s + 2 * hh + e / 8, q = e % 8;
            const int c = g / kK, p = g % kK;
            const signed char v = dig[((size_t)n * K + ((size_t)c * kK + p) * kK + q) * 3 + d];
            word |= (uint32_t)(uint8_t)v << (8 * e4);
          }
          wpk[((size_t)(s * 3 + d) * 4 + wq) * 64 + lane] = (int)word;
        }
}

hipError_t launch_conv1_i8(const ConvLayer& L, int B, const uint8_t* obs, const int* wpk,
                           const float* scale, const float* bpk, void* out, int out_bf16,
                           int planes, int waves_hint, int image, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (planes != 2 && planes != 3) return hipErrorInvalidValue;
  const int n_xchunks = (L.Wo + 31) / 32;
  const int frame_bytes = L.cin * L.H * L.W;
  // The frame-resident variant pays from four frames per workgroup on (measured on MI355X:
  // B = 4096 bf16 68.5 -> 58.5 us, B = 2048 fp32 52.8 -> 41.4 us, B = 1024 fp32 22.3 -> 23.8 us);
  // both variants give the same bits, so the choice may depend on the batch of the call.
  if (image && B >= 2048 && n_xchunks == 1 && frame_bytes % 16 == 0 &&
      frame_bytes <= 7 * 256 * 16 && ((uintptr_t)obs & 15) == 0 && L.cin == 3) {
    // two workgroups per CU, each walking its share of the frames
    const int blocks = B < 512 ? B : 512;
    const size_t lds = (size_t)frame_bytes;
#define SF_LAUNCH_IMG(BF, ND)                                            \
  conv1_u8_i8_image_kernel<3, BF, ND><<<blocks, 64 * kWaves, lds, st>>>( \
      obs, wpk, scale, bpk, out, B, L.H, L.W, L.Ho, L.Wo)
    if (out_bf16) {
      if (planes == 2) SF_LAUNCH_IMG(true, 2); else SF_LAUNCH_IMG(true, 3);
    } else {
      if (planes == 2) SF_LAUNCH_IMG(false, 2); else SF_LAUNCH_IMG(false, 3);
    }
#undef SF_LAUNCH_IMG
    return hipGetLastError();
  }
  const long long n_items = (long long)B * L.Ho * n_xchunks;
  long long waves = waves_hint > 0 ? waves_hint : 2048;  // two wavefronts per SIMD on 256 CUs
  if (waves > n_items) waves = n_items;
  const int blocks = (int)((waves + kWaves - 1) / kWaves);
  const int n_waves_total = blocks * kWaves;
#define SF_LAUNCH_K(C, BF, ND)                                      \
  conv1_u8_i8_kernel<C, BF, ND><<<blocks, 64 * kWaves, 0, st>>>(    \
      obs, wpk, scale, bpk, out, L.H, L.W, L.Ho, L.Wo, n_xchunks, n_items, n_waves_total)
#define SF_LAUNCH_CIN(C)                                                      \
  do {                                                                        \
    if (out_bf16) {                                                           \
      if (planes == 2) SF_LAUNCH_K(C, true, 2); else SF_LAUNCH_K(C, true, 3); \
    } else {                                                                  \
      if (planes == 2) SF_LAUNCH_K(C, false, 2); else SF_LAUNCH_K(C, false, 3); \
    }                                                                         \
  } while (0)
  switch (L.cin) {
    case 1: SF_LAUNCH_CIN(1); break;
    case 3: SF_LAUNCH_CIN(3); break;
    case 4: SF_LAUNCH_CIN(4); break;
    default: return hipErrorInvalidValue;
  }
#undef SF_LAUNCH_CIN
#undef SF_LAUNCH_K
  return hipGetLastError();
}

}  // namespace sf

// 3x3 / stride 1 / pad 1 convolutions of the residual encoder on the 16-bit MFMA with
// LDS-staged input tiles (the residual encoder follows IMPALA; paper, App. DMLab-30).
//
// A workgroup owns a TH x TWW block of output pixels of one frame.  It stages the
// (TH+2) x (TWW+2) input patch in LDS once, as 16-bit channels-last pixels (converted
// from fp32 and ReLU'd on the way where the layer asks for it; pixels outside the
// image are zero), so every input value is fetched from memory once per tile instead
// of once per filter tap.  The nine taps then read their operands straight out of the
// patch: for tap (p, q) the B operand of output pixel (y, x) is the 16-byte run of 8
// channels at patch[y+p][x+q].  The whole filter bank (9 taps x Cin x 32 channels) is
// resident in each wave's registers as A operands.  There is no K loop and a single
// barrier.
//
// v_mfma_f32_32x32x16_{f16,bf16}: lane l supplies A[i = l%32][k = 8*(l/32) + e] and
// B[k = 8*(l/32) + e][j = l%32].  A = weights (i = output channel), B = pixels
// (j = pixel of the wave's 32-pixel tile), so D[i][j] leaves a lane with 4 consecutive
// channels of one pixel per register quad: 8- or 16-byte stores, fused bias, residual
// add (fp32 stream) and ReLU.
//
// The first convolution of the encoder reads planar bytes: its patch holds normalised
// 16-bit pixels of 3 channels padded to 4 (8 bytes per pixel), K is ordered (filter
// row; filter column padded to 4; channel padded to 4) so that one MFMA (K = 16)
// covers one filter row and a lane's operand is the 16-byte run of two neighbouring
// patch pixels.
#include <string.h>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <bool kF16>
__device__ inline unsigned to_h(float f) {
  if (kF16) return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);
  unsigned u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
template <bool kF16>
__device__ inline float from_h(unsigned h) {
  if (kF16) return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
  return __uint_as_float(h << 16);
}
__device__ inline unsigned relu_h2(unsigned w) {
  unsigned neg = (w >> 15) & 0x00010001u;
  return w & ~(neg * 0xFFFFu);
}
template <bool kF16>
__device__ inline f32x16 mfma16(u32x4 a, u32x4 b, f32x16 c) {
  if (kF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

struct PatchArgs {
  const void* in;      // fp32 or 16-bit [B][H][W][CIN]
  const u32x4* wpk;    // [9][CIN/16][64] A operands
  const float* bias;   // [32]
  const void* resid;   // fp32 or 16-bit [B][H][W][N], or null
  void* out;           // 16-bit or fp32 [B][H][W][N]
  int B, H, W, N;
  int tiles_x, tiles_y;
  int in_f32, relu_in, relu_out, out_f32, resid_f32;
};

// TWW: tile width in pixels (16 or 32); a wave's 32-pixel MFMA tile is 32/TWW rows
// high; RPW such tiles per wave, four waves stacked vertically.
template <int CIN, int TWW, int RPW, bool kF16>
__global__ __launch_bounds__(256) void conv3x3_patch_kernel(PatchArgs g) {
  constexpr int RW = 32 / TWW;          // rows of one MFMA tile
  constexpr int TH = 4 * RPW * RW;      // rows of the workgroup tile
  constexpr int PH = TH + 2, PW = TWW + 2;
  constexpr int PITCH = CIN * 2 + 16;   // bytes per patch pixel: conflict-free 16-byte reads
  constexpr int C8 = CIN / 8;
  constexpr int NS = CIN / 16;          // MFMA K steps per tap
  __shared__ __attribute__((aligned(16))) unsigned char patch[PH * PW * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  int t = blockIdx.x;
  const int tx = t % g.tiles_x;
  t /= g.tiles_x;
  const int ty = t % g.tiles_y;
  const int b = t / g.tiles_y;
  const int y0 = ty * TH, x0 = tx * TWW;

  // filter bank -> registers (in flight while the patch is staged)
  u32x4 wreg[9][NS];
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int s = 0; s < NS; ++s) wreg[tap][s] = g.wpk[(tap * NS + s) * 64 + lane];

  // stage the input patch
  const size_t img = (size_t)b * g.H * g.W * CIN;
  for (int idx = tid; idx < PH * PW * C8; idx += 256) {
    const int pix = idx / C8, c8 = idx - pix * C8;
    const int py = pix / PW, px = pix - py * PW;
    const int y = y0 - 1 + py, x = x0 - 1 + px;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (y >= 0 && y < g.H && x >= 0 && x < g.W) {
      const size_t e = img + ((size_t)y * g.W + x) * CIN + c8 * 8;
      if (g.in_f32) {
        const f32x4 lo = *(const f32x4*)((const float*)g.in + e);
        const f32x4 hi = *(const f32x4*)((const float*)g.in + e + 4);
        v[0] = to_h<kF16>(lo[0]) | (to_h<kF16>(lo[1]) << 16);
        v[1] = to_h<kF16>(lo[2]) | (to_h<kF16>(lo[3]) << 16);
        v[2] = to_h<kF16>(hi[0]) | (to_h<kF16>(hi[1]) << 16);
        v[3] = to_h<kF16>(hi[2]) | (to_h<kF16>(hi[3]) << 16);
      } else {
        v = *(const u32x4*)((const uint16_t*)g.in + e);
      }
      if (g.relu_in) {
        v[0] = relu_h2(v[0]);
        v[1] = relu_h2(v[1]);
        v[2] = relu_h2(v[2]);
        v[3] = relu_h2(v[3]);
      }
    }
    *(u32x4*)(patch + pix * PITCH + c8 * 16) = v;
  }
  __syncthreads();

#pragma unroll
  for (int rt = 0; rt < RPW; ++rt) {
    const int ry = (wave * RPW + rt) * RW + li / TWW;  // row inside the workgroup tile
    const int cx = li % TWW;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    const unsigned char* base = patch + (ry * PW + cx) * PITCH + lh * 16;
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
      for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const u32x4 frag = *(const u32x4*)(base + (p * PW + q) * PITCH + s * 32);
          acc = mfma16<kF16>(wreg[p * 3 + q][s], frag, acc);
        }
    // epilogue: D[i][j], i = channel = (v%4) + 4*lh + 8*(v/4), j = pixel = li
    const int y = y0 + ry, x = x0 + cx;
    if (y < g.H && x < g.W) {
      const size_t o = (((size_t)b * g.H + y) * g.W + x) * g.N;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int ch = 8 * q4 + 4 * lh;
        if (ch >= g.N) continue;
        float r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = acc[4 * q4 + u] + g.bias[ch + u];
        if (g.resid) {
          if (g.resid_f32) {
            const f32x4 rv = *(const f32x4*)((const float*)g.resid + o + ch);
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] += rv[u];
          } else {
            const u32x2 rv = *(const u32x2*)((const uint16_t*)g.resid + o + ch);
            r[0] += from_h<kF16>(rv[0] & 0xFFFFu);
            r[1] += from_h<kF16>(rv[0] >> 16);
            r[2] += from_h<kF16>(rv[1] & 0xFFFFu);
            r[3] += from_h<kF16>(rv[1] >> 16);
          }
        }
        if (g.relu_out) {
#pragma unroll
          for (int u = 0; u < 4; ++u) r[u] = fmaxf(r[u], 0.0f);
        }
        if (g.out_f32) {
          const f32x4 ov = {r[0], r[1], r[2], r[3]};
          *(f32x4*)((float*)g.out + o + ch) = ov;
        } else {
          u32x2 ov;
          ov[0] = to_h<kF16>(r[0]) | (to_h<kF16>(r[1]) << 16);
          ov[1] = to_h<kF16>(r[2]) | (to_h<kF16>(r[3]) << 16);
          *(u32x2*)((uint16_t*)g.out + o + ch) = ov;
        }
      }
    }
  }
}

struct StemArgs {
  const uint8_t* obs;  // planar bytes [B][3][H][W]
  const u32x4* wpk;    // [3 filter rows][64] A operands
  const float* bias;   // [32]
  uint16_t* out;       // 16-bit [B][H][W][N]
  int B, H, W, N;
  int tiles_x, tiles_y;
  float obs_sub, obs_mul;
};

// First convolution of the encoder: 3 byte planes in, N = 16 or 32 channels out.
// 32 x (8 rows) pixel tile per workgroup, two 32-pixel rows per wave.
template <bool kF16>
__global__ __launch_bounds__(256) void conv3x3_stem_kernel(StemArgs g) {
  constexpr int TWW = 32, RPW = 2, TH = 4 * RPW;
  constexpr int PH = TH + 2, PW = TWW + 4;  // columns x0-1 .. x0+34 (the 4th, phantom tap reads x+2)
  __shared__ __attribute__((aligned(16))) unsigned char patch[PH * PW * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  int t = blockIdx.x;
  const int tx = t % g.tiles_x;
  t /= g.tiles_x;
  const int ty = t % g.tiles_y;
  const int b = t / g.tiles_y;
  const int y0 = ty * TH, x0 = tx * TWW;

  u32x4 wreg[3];
#pragma unroll
  for (int p = 0; p < 3; ++p) wreg[p] = g.wpk[p * 64 + lane];

  const uint8_t* frame = g.obs + (size_t)b * 3 * g.H * g.W;
  for (int pix = tid; pix < PH * PW; pix += 256) {
    const int py = pix / PW, px = pix - py * PW;
    const int y = y0 - 1 + py, x = x0 - 1 + px;
    u32x2 v = {0u, 0u};
    if (y >= 0 && y < g.H && x >= 0 && x < g.W) {
      const size_t o = (size_t)y * g.W + x;
      const float c0 = ((float)frame[o] - g.obs_sub) * g.obs_mul;
      const float c1 = ((float)frame[o + (size_t)g.H * g.W] - g.obs_sub) * g.obs_mul;
      const float c2 = ((float)frame[o + 2 * (size_t)g.H * g.W] - g.obs_sub) * g.obs_mul;
      v[0] = to_h<kF16>(c0) | (to_h<kF16>(c1) << 16);
      v[1] = to_h<kF16>(c2);
    }
    *(u32x2*)(patch + pix * 8) = v;
  }
  __syncthreads();

#pragma unroll
  for (int rt = 0; rt < RPW; ++rt) {
    const int ry = wave * RPW + rt;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    // lane half lh covers filter columns 2*lh and 2*lh+1: patch pixels x-1+2*lh, x+2*lh
    const unsigned char* base = patch + (ry * PW + li + 2 * lh) * 8;
#pragma unroll
    for (int p = 0; p < 3; ++p) {
      const u32x2 a0 = *(const u32x2*)(base + p * PW * 8);
      const u32x2 a1 = *(const u32x2*)(base + p * PW * 8 + 8);
      const u32x4 frag = {a0[0], a0[1], a1[0], a1[1]};
      acc = mfma16<kF16>(wreg[p], frag, acc);
    }
    const int y = y0 + ry, x = x0 + li;
    if (y < g.H && x < g.W) {
      const size_t o = (((size_t)b * g.H + y) * g.W + x) * g.N;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int ch = 8 * q4 + 4 * lh;
        if (ch >= g.N) continue;
        u32x2 ov;
        ov[0] = to_h<kF16>(acc[4 * q4 + 0] + g.bias[ch + 0]) |
                (to_h<kF16>(acc[4 * q4 + 1] + g.bias[ch + 1]) << 16);
        ov[1] = to_h<kF16>(acc[4 * q4 + 2] + g.bias[ch + 2]) |
                (to_h<kF16>(acc[4 * q4 + 3] + g.bias[ch + 3]) << 16);
        *(u32x2*)(g.out + o + ch) = ov;
      }
    }
  }
}

// fp32 -> fp16 bits, round to nearest even, subnormals kept.
uint16_t host_f32_to_f16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  const uint32_t sign = (u >> 16) & 0x8000u;
  const int32_t exp = (int32_t)((u >> 23) & 0xFF) - 127 + 15;
  uint32_t man = u & 0x7FFFFFu;
  if (((u >> 23) & 0xFF) == 0xFF) return (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0));
  if (exp >= 31) return (uint16_t)(sign | 0x7C00u);
  if (exp <= 0) {
    if (exp < -10) return (uint16_t)sign;
    man |= 0x800000u;
    const int shift = 14 - exp;
    uint32_t h = man >> shift;
    const uint32_t remb = man & ((1u << shift) - 1), half = 1u << (shift - 1);
    if (remb > half || (remb == half && (h & 1))) ++h;
    return (uint16_t)(sign | h);
  }
  uint32_t h = ((uint32_t)exp << 10) | (man >> 13);
  const uint32_t remb = man & 0x1FFFu;
  if (remb > 0x1000u || (remb == 0x1000u && (h & 1))) ++h;
  return (uint16_t)(sign | h);
}

// the bf16 value of a weight, as bf16 bits or (the same value) as fp16 bits
uint16_t weight_bits(float v, bool f16) {
  uint32_t u;
  memcpy(&u, &v, 4);
  u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
  if (!f16) return (uint16_t)(u >> 16);
  float bv;
  memcpy(&bv, &u, 4);
  return host_f32_to_f16(bv);
}

template <int CIN, int TWW, int RPW>
hipError_t launch_patch(const PatchArgs& a, bool f16, hipStream_t st) {
  PatchArgs g = a;
  constexpr int TH = 4 * RPW * (32 / TWW);
  g.tiles_x = (g.W + TWW - 1) / TWW;
  g.tiles_y = (g.H + TH - 1) / TH;
  const long long blocks = (long long)g.B * g.tiles_x * g.tiles_y;
  if (f16)
    conv3x3_patch_kernel<CIN, TWW, RPW, true><<<(unsigned)blocks, 256, 0, st>>>(g);
  else
    conv3x3_patch_kernel<CIN, TWW, RPW, false><<<(unsigned)blocks, 256, 0, st>>>(g);
  return hipGetLastError();
}

}  // namespace

bool conv3x3_patch_supported(int cin, int cout, int k, int stride, int pad) {
  return k == 3 && stride == 1 && pad == 1 && (cin == 16 || cin == 32) && (cout == 16 || cout == 32);
}

// A operands of the patch kernel: wpk[((tap*NS + s)*64 + lane)*8 + e] =
// w[n = lane%32][c = 16*s + 8*(lane/32) + e][p][q], tap = 3*p + q; zero for n >= cout.
void conv3x3_patch_pack(const float* w, const float* bias, int cout, int cin, bool f16,
                        std::vector<uint16_t>& wpk, std::vector<float>& b32) {
  const int ns = cin / 16;
  wpk.assign((size_t)9 * ns * 64 * 8, 0);
  b32.assign(32, 0.0f);
  for (int n = 0; n < cout; ++n) b32[n] = bias[n];
  for (int tap = 0; tap < 9; ++tap)
    for (int s = 0; s < ns; ++s)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int n = lane & 31, c = 16 * s + 8 * (lane >> 5) + e, p = tap / 3, q = tap % 3;
          if (n < cout)
            wpk[(((size_t)tap * ns + s) * 64 + lane) * 8 + e] =
                weight_bits(w[(((size_t)n * cin + c) * 3 + p) * 3 + q], f16);
        }
}

hipError_t launch_conv3x3_patch(const void* in, const uint16_t* wpk, const float* bias32,
                                const void* resid, int resid_f32, void* out, int B, int H, int W,
                                int cin, int cout, int in_f32, int relu_in, int relu_out,
                                int out_f32, int f16, hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  PatchArgs g;
  g.in = in; g.wpk = (const u32x4*)wpk; g.bias = bias32; g.resid = resid; g.out = out;
  g.B = B; g.H = H; g.W = W; g.N = cout;
  g.tiles_x = g.tiles_y = 0;
  g.in_f32 = in_f32; g.relu_in = relu_in; g.relu_out = relu_out; g.out_f32 = out_f32;
  g.resid_f32 = resid_f32;
  const bool wide = W > 16;            // 32-pixel-wide tiles unless the image is narrow
  const bool tall = H % 12 == 0 && wide;  // three row tiles per wave when they divide the height
  if (cin == 16) {
    if (!wide) return launch_patch<16, 16, 1>(g, f16 != 0, st);
    return tall ? launch_patch<16, 32, 3>(g, f16 != 0, st) : launch_patch<16, 32, 1>(g, f16 != 0, st);
  }
  if (cin == 32) {
    if (!wide) return launch_patch<32, 16, 1>(g, f16 != 0, st);
    return tall ? launch_patch<32, 32, 3>(g, f16 != 0, st) : launch_patch<32, 32, 1>(g, f16 != 0, st);
  }
  return hipErrorInvalidValue;
}

// (for the packers of the other residual-encoder kernels)
uint16_t conv_weight_bits(float v, bool f16) { return weight_bits(v, f16); }

bool conv3x3_stem_supported(int cin, int cout) { return cin == 3 && (cout == 16 || cout == 32); }

// A operands of the stem kernel: wpk[(p*64 + lane)*8 + e] = w[n][c = e%4][p][q = 2*(lane/32) + e/4]
// for c < 3 and q < 3, else zero.
void conv3x3_stem_pack(const float* w, const float* bias, int cout, bool f16,
                       std::vector<uint16_t>& wpk, std::vector<float>& b32) {
  wpk.assign((size_t)3 * 64 * 8, 0);
  b32.assign(32, 0.0f);
  for (int n = 0; n < cout; ++n) b32[n] = bias[n];
  for (int p = 0; p < 3; ++p)
    for (int lane = 0; lane < 64; ++lane)
      for (int e = 0; e < 8; ++e) {
        const int n = lane & 31, c = e % 4, q = 2 * (lane >> 5) + e / 4;
        if (n < cout && c < 3 && q < 3)
          wpk[((size_t)p * 64 + lane) * 8 + e] = weight_bits(w[(((size_t)n * 3 + c) * 3 + p) * 3 + q], f16);
      }
}

hipError_t launch_conv3x3_stem(const uint8_t* obs, const uint16_t* wpk, const float* bias32, void* out,
                               int B, int H, int W, int cout, float obs_sub, float obs_mul, int f16,
                               hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  StemArgs g;
  g.obs = obs; g.wpk = (const u32x4*)wpk; g.bias = bias32; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.N = cout;
  g.tiles_x = (W + 31) / 32;
  g.tiles_y = (H + 7) / 8;
  g.obs_sub = obs_sub; g.obs_mul = obs_mul;
  const long long blocks = (long long)B * g.tiles_x * g.tiles_y;
  if (f16)
    conv3x3_stem_kernel<true><<<(unsigned)blocks, 256, 0, st>>>(g);
  else
    conv3x3_stem_kernel<false><<<(unsigned)blocks, 256, 0, st>>>(g);
  return hipGetLastError();
}

}  // namespace sf

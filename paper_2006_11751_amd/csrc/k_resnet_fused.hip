// Fused kernels of the residual encoder (the encoder follows IMPALA; paper, App. DMLab-30),
// fp16 activations, 16-bit MFMA with fp32 accumulation.
//
//   conv3x3_pool_kernel   stage convolution (3x3, stride 1, pad 1, + bias) and the 3x3 /
//                         stride 2 / pad 1 max-pool behind it.  The full-resolution
//                         convolution output lives only in LDS: the workgroup computes
//                         the (2*PTH+1) x (2*PTW+1) convolution pixels that its PTH x PTW
//                         pooled pixels look at (one halo row and column are recomputed
//                         per tile), rounds them to fp16 exactly as the unfused pair of
//                         kernels does, and pools out of LDS.
//   res_block_kernel      one residual block, y = x + conv_b(relu(conv_a(relu(x)))): the
//                         branch tensor between the two convolutions lives only in LDS
//                         (a one-pixel halo of it is recomputed per tile).
//
// Both use the operand scheme of the unfused patch kernels: the input patch is staged in
// LDS once as channels-last fp16 pixels (pitch 2*C + 16 bytes, so the 16-byte operand reads
// of 32 neighbouring pixels do not collide), the whole filter bank sits in registers as A
// operands, and for filter tap (p, q) the B operand of output pixel (y, x) is the 16-byte
// run of 8 channels at patch[y+p][x+q].  The pixels of a region are enumerated in row-major
// order over its in-image part only and cut into 32-pixel MFMA tiles, so tiles at the image
// border do no work for pixels outside the image.
//
// v_mfma_f32_32x32x16_f16: lane l supplies A[i = l%32][k = 8*(l/32) + e] and
// B[k = 8*(l/32) + e][j = l%32]; D[i][j] sits in lane j + 32*((i/4)%2), register
// (i%4) + 4*(i/8).  A = weights (i = output channel), B = pixels.
#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ inline unsigned f16_bits(float f) {
  return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);
}
__device__ inline unsigned pack_f16(float a, float b) { return f16_bits(a) | (f16_bits(b) << 16); }
__device__ inline float f16_value(unsigned h) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
__device__ inline unsigned max_h2(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(f16x2, a),
                                                                __builtin_bit_cast(f16x2, b)));
}
// ReLU of two packed fp16 values
__device__ inline unsigned relu_h2(unsigned w) { return max_h2(w, 0u); }
__device__ inline f32x16 mfma_f16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by block id.  This
// maps block id -> tile index so that each XCD works through one contiguous run of tiles:
// neighbouring tiles of a frame, which share halo pixels, then meet in the same L2.
__device__ inline int xcd_contiguous_tile(int bid, int nblocks) {
  const int per = nblocks >> 3, rem = nblocks & 7;
  const int xcd = bid & 7, idx = bid >> 3;
  return xcd * per + min(xcd, rem) + idx;
}

// Stages the PH x PW pixel patch whose pixel (0, 0) is image pixel (ya, xa) of an fp16
// channels-last image; pixels outside the image are zero.  All of a thread's loads are
// issued before the first of them is consumed.
template <int C, int PITCH, int NT, int PH, int PW>
__device__ inline void stage_patch(unsigned char* patch, const uint16_t* img, int H, int W, int ya,
                                   int xa, bool relu, int tid) {
  constexpr int C8 = C / 8;
  constexpr int TOTAL = PH * PW * C8;
  constexpr int ITERS = (TOTAL + NT - 1) / NT;
  u32x4 v[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int idx = tid + it * NT;
    const int pix = idx / C8, c8 = idx - pix * C8;
    const int py = pix / PW, px = pix - py * PW;
    const int y = ya + py, x = xa + px;
    // branch-free: load from the nearest in-image pixel, then blank what lies outside
    const bool inside = idx < TOTAL && y >= 0 && y < H && x >= 0 && x < W;
    const int yc = min(max(y, 0), H - 1), xc = min(max(x, 0), W - 1);
    v[it] = *(const u32x4*)(img + ((size_t)yc * W + xc) * C + c8 * 8);
    if (!inside) v[it] = u32x4{0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int idx = tid + it * NT;
    const int pix = idx / C8, c8 = idx - pix * C8;
    if (relu) {
      v[it][0] = relu_h2(v[it][0]);
      v[it][1] = relu_h2(v[it][1]);
      v[it][2] = relu_h2(v[it][2]);
      v[it][3] = relu_h2(v[it][3]);
    }
    if (idx < TOTAL) *(u32x4*)(patch + pix * PITCH + c8 * 16) = v[it];
  }
}

// The 9 * C/16 MFMAs of N independent 32-pixel tiles, interleaved so that consecutive
// MFMAs do not depend on each other.  base[n] points at the lane's pixel of tile n (tap
// (0, 0)) plus the lane half's 16-byte channel offset; PWP = patch pitch in pixels; the
// accumulators start from init (the bias in the D layout).
template <int C, int PITCH, int N>
__device__ inline void conv_taps(const u32x4 (&wreg)[9][C / 16], const unsigned char* (&base)[N],
                                 int PWP, const f32x16& init, f32x16 (&acc)[N]) {
#pragma unroll
  for (int n = 0; n < N; ++n) acc[n] = init;
#pragma unroll
  for (int p = 0; p < 3; ++p)
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int s = 0; s < C / 16; ++s)
#pragma unroll
        for (int n = 0; n < N; ++n) {
          const u32x4 frag = *(const u32x4*)(base[n] + (p * PWP + q) * PITCH + s * 32);
          acc[n] = mfma_f16(wreg[p * 3 + q][s], frag, acc[n]);
        }
}

// Pixel of lane li in 32-pixel tile `tile` of a region whose in-image part has npix pixels
// in rows of ncols, starting at region row r_off and column c_off.  Lanes past the end
// repeat the last pixel and are not live.
struct TilePixel {
  int ry, cx;
  bool live;
};
// inv_ncols = 1.0f / ncols: (n + 0.5) * inv_ncols truncates to n / ncols exactly for the
// few thousand pixels of a region.
__device__ inline TilePixel tile_pixel(int tile, int li, int npix, int ncols, float inv_ncols,
                                       int r_off, int c_off) {
  const int n = tile * 32 + li;
  TilePixel t;
  t.live = n < npix;
  const int nc = t.live ? n : npix - 1;
  t.ry = (int)(((float)nc + 0.5f) * inv_ncols);
  t.cx = nc - t.ry * ncols + c_off;
  t.ry += r_off;
  return t;
}

template <int N>
struct Count {
  static constexpr int value = N;
};

// A wave's tiles (wave, wave + NW, ...) two at a time, then the odd one.
template <int NW, typename F>
__device__ inline void for_wave_tiles(int wave, int npix, F&& f) {
  int tile = wave;
  for (; (tile + NW) * 32 < npix; tile += 2 * NW) f(Count<2>(), tile);
  if (tile * 32 < npix) f(Count<1>(), tile);
}

struct ConvPoolArgs {
  const void* in;      // stem: planar bytes [B][3][H][W]; else fp16 [B][H][W][CIN]
  const u32x4* wpk;    // A operands (stem: [3][64]; else [9][CIN/16][64])
  const float* bias;   // [32]
  uint16_t* out;       // fp16 [B][Ho][Wo][COUT]
  int B, H, W, Ho, Wo;
  int tiles_x, tiles_y;
  float obs_sub, obs_mul;
};

// CIN == 3: the encoder's first convolution (bytes in, normalised on the way into LDS;
// requires W % 4 == 0).  PTH x PTW pooled pixels per workgroup, NW waves.
template <int CIN, int COUT, int PTH, int PTW, int NW>
__global__ __launch_bounds__(64 * NW) void conv3x3_pool_kernel(ConvPoolArgs g) {
  constexpr bool STEM = CIN == 3;
  constexpr int NT = 64 * NW;
  constexpr int CH = 2 * PTH + 1, CW = 2 * PTW + 1;  // convolution region
  constexpr int PH = CH + 2;
  // Patch column 0 is image column cc0 - XOFF.  The stem patch starts 3 columns further
  // left so that it begins on a 4-byte boundary of the byte planes, and extends one
  // column further right for the zero-weight fourth filter column of its K layout.
  constexpr int XOFF = STEM ? 3 : 1;
  constexpr int PW = STEM ? (CW + 5 + 3) / 4 * 4 : CW + 2;
  constexpr int PITCH = STEM ? 8 : CIN * 2 + 16;
  constexpr int CP = COUT * 2 + 8;  // bytes per pixel of the convolution buffer
  constexpr int NS = STEM ? 1 : CIN / 16;
  __shared__ __attribute__((aligned(16))) unsigned char patch[PH * PW * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char cbuf[CH * CW * CP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  int t = xcd_contiguous_tile(blockIdx.x, gridDim.x);
  const int tx = t % g.tiles_x;
  t /= g.tiles_x;
  const int ty = t % g.tiles_y;
  const int b = t / g.tiles_y;
  const int oy0 = ty * PTH, ox0 = tx * PTW;
  const int cr0 = 2 * oy0 - 1, cc0 = 2 * ox0 - 1;  // first convolution row / column of the region

  u32x4 wreg[STEM ? 3 : 9][NS];
#pragma unroll
  for (int tap = 0; tap < (STEM ? 3 : 9); ++tap)
#pragma unroll
    for (int s = 0; s < NS; ++s) wreg[tap][s] = g.wpk[(tap * NS + s) * 64 + lane];

  if constexpr (STEM) {
    const uint8_t* frame = (const uint8_t*)g.in + (size_t)b * 3 * g.H * g.W;
    const size_t plane = (size_t)g.H * g.W;
    constexpr int Q = PW / 4;
    constexpr int ITERS = (PH * Q + NT - 1) / NT;
    uint32_t w[ITERS][3];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int i = tid + it * NT;
      const int py = i / Q, j = i - py * Q;
      const int y = cr0 - 1 + py, x4 = cc0 - XOFF + 4 * j;
      w[it][0] = w[it][1] = w[it][2] = 0u;
      if (i < PH * Q && y >= 0 && y < g.H && x4 >= 0 && x4 < g.W) {
        const size_t o = (size_t)y * g.W + x4;
        w[it][0] = *(const uint32_t*)(frame + o);
        w[it][1] = *(const uint32_t*)(frame + plane + o);
        w[it][2] = *(const uint32_t*)(frame + 2 * plane + o);
      }
    }
    // (a pixel outside the image is zero, not the normalised value of byte 0)
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int i = tid + it * NT;
      const int py = i / Q, j = i - py * Q;
      const int y = cr0 - 1 + py, x4 = cc0 - XOFF + 4 * j;
      const bool inside = y >= 0 && y < g.H && x4 >= 0 && x4 < g.W;
      u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
      if (inside) {
        float c[4][3];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
          for (int ch = 0; ch < 3; ++ch)
            c[k][ch] = ((float)((w[it][ch] >> (8 * k)) & 0xFFu) - g.obs_sub) * g.obs_mul;
        lo[0] = pack_f16(c[0][0], c[0][1]); lo[1] = f16_bits(c[0][2]);
        lo[2] = pack_f16(c[1][0], c[1][1]); lo[3] = f16_bits(c[1][2]);
        hi[0] = pack_f16(c[2][0], c[2][1]); hi[1] = f16_bits(c[2][2]);
        hi[2] = pack_f16(c[3][0], c[3][1]); hi[3] = f16_bits(c[3][2]);
      }
      if (i < PH * Q) {
        u32x4* dst = (u32x4*)(patch + (py * PW + 4 * j) * 8);
        dst[0] = lo;
        dst[1] = hi;
      }
    }
  } else {
    stage_patch<CIN, PITCH, NT, PH, PW>(patch, (const uint16_t*)g.in + (size_t)b * g.H * g.W * CIN,
                                        g.H, g.W, cr0 - 1, cc0 - 1, false, tid);
  }
  __syncthreads();

  // the bias in the accumulator layout: register 4*q4 + u holds channel 8*q4 + 4*lh + u
  f32x16 bias_acc;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 bv = *(const f32x4*)(g.bias + 8 * q4 + 4 * lh);
#pragma unroll
    for (int u = 0; u < 4; ++u) bias_acc[4 * q4 + u] = bv[u];
  }

  // in-image part of the region
  const int r_off = cr0 < 0 ? 1 : 0, c_off = cc0 < 0 ? 1 : 0;
  const int nrows = min(CH, g.H - cr0) - r_off, ncols = min(CW, g.W - cc0) - c_off;
  const int npix = nrows * ncols;
  const float inv_ncols = 1.0f / (float)ncols;
  for_wave_tiles<NW>(wave, npix, [&](auto cnt, int tile) {
    constexpr int N = decltype(cnt)::value;
    TilePixel tp[N];
    f32x16 acc[N];
#pragma unroll
    for (int n = 0; n < N; ++n) tp[n] = tile_pixel(tile + n * NW, li, npix, ncols, inv_ncols, r_off, c_off);
    if constexpr (STEM) {
#pragma unroll
      for (int n = 0; n < N; ++n) acc[n] = bias_acc;
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int n = 0; n < N; ++n) {
          // lane half lh covers filter columns 2*lh and 2*lh+1
          const unsigned char* base = patch + ((tp[n].ry + p) * PW + tp[n].cx + XOFF - 1 + 2 * lh) * 8;
          const u32x2 a0 = *(const u32x2*)base;
          const u32x2 a1 = *(const u32x2*)(base + 8);
          const u32x4 frag = {a0[0], a0[1], a1[0], a1[1]};
          acc[n] = mfma_f16(wreg[p][0], frag, acc[n]);
        }
    } else {
      const unsigned char* base[N];
#pragma unroll
      for (int n = 0; n < N; ++n) base[n] = patch + (tp[n].ry * PW + tp[n].cx) * PITCH + lh * 16;
      conv_taps<CIN, PITCH, N>(wreg, base, PW, bias_acc, acc);
    }
#pragma unroll
    for (int n = 0; n < N; ++n) {
      if (!tp[n].live) continue;
      unsigned char* dst = cbuf + (tp[n].ry * CW + tp[n].cx) * CP;
#pragma unroll
      for (int q4 = 0; q4 < COUT / 8; ++q4) {
        const int ch = 8 * q4 + 4 * lh;
        u32x2 ov;
        ov[0] = pack_f16(acc[n][4 * q4 + 0], acc[n][4 * q4 + 1]);
        ov[1] = pack_f16(acc[n][4 * q4 + 2], acc[n][4 * q4 + 3]);
        *(u32x2*)(dst + ch * 2) = ov;
      }
    }
  });
  // Region pixels outside the image were not computed: they are the pool's padding, -inf.
  if (cr0 < 0 || cc0 < 0 || cr0 + CH > g.H || cc0 + CW > g.W) {  // uniform: border tiles only
    for (int i = tid; i < CH * CW; i += NT) {
      const int ry = i / CW, cx = i - ry * CW;
      const int r = cr0 + ry, cc = cc0 + cx;
      if (r < 0 || r >= g.H || cc < 0 || cc >= g.W) {
        const u32x2 ninf = {0xFC00FC00u, 0xFC00FC00u};
#pragma unroll
        for (int c4 = 0; c4 < COUT / 4; ++c4) *(u32x2*)(cbuf + i * CP + c4 * 8) = ninf;
      }
    }
  }
  __syncthreads();

  // 3x3 / stride 2 / pad 1 max-pool out of LDS: pooled (oy, ox) covers convolution rows
  // 2*oy-1 .. 2*oy+1 and columns 2*ox-1 .. 2*ox+1 (region rows 2*py .. 2*py+2).
  constexpr int C4 = COUT / 4;
  for (int i = tid; i < PTH * PTW * C4; i += NT) {
    const int pp = i / C4, c4 = i - pp * C4;
    const int py = pp / PTW, px = pp - py * PTW;
    const int oy = oy0 + py, ox = ox0 + px;
    if (oy >= g.Ho || ox >= g.Wo) continue;
    const unsigned char* win = cbuf + (2 * py * CW + 2 * px) * CP + c4 * 8;
    u32x2 v[9];
#pragma unroll
    for (int dy = 0; dy < 3; ++dy)
#pragma unroll
      for (int dx = 0; dx < 3; ++dx) v[dy * 3 + dx] = *(const u32x2*)(win + (dy * CW + dx) * CP);
    unsigned m0 = v[0][0], m1 = v[0][1];
#pragma unroll
    for (int k = 1; k < 9; ++k) {
      m0 = max_h2(m0, v[k][0]);
      m1 = max_h2(m1, v[k][1]);
    }
    const u32x2 ov = {m0, m1};
    *(u32x2*)(g.out + (((size_t)b * g.Ho + oy) * g.Wo + ox) * COUT + 4 * c4) = ov;
  }
}

struct BlockArgs {
  const uint16_t* x;    // fp16 [B][H][W][C]
  const u32x4* wa;      // conv_a A operands [9][C/16][64]
  const u32x4* wb;      // conv_b
  const float* ba;      // [32]
  const float* bb;      // [32]
  uint16_t* out;        // fp16 [B][H][W][C]
  int B, H, W;
  int tiles_x, tiles_y;
  int relu_out;
};

// One residual block on a TH x TW pixel tile.  The x patch (two-pixel halo) is staged with
// the block's leading ReLU applied; the branch tensor t = relu(conv_a + bias) is produced
// on the tile plus a one-pixel halo (zero outside the image, as conv_b's padding wants it)
// into LDS; conv_b reads it from there and adds bias and the un-rectified x from memory.
template <int C, int TH, int TW, int NW>
__global__ __launch_bounds__(64 * NW, C == 32 ? 3 : 1) void res_block_kernel(BlockArgs g) {
  constexpr int NT = 64 * NW;
  constexpr int XH = TH + 4, XW = TW + 4;  // x patch
  constexpr int UH = TH + 2, UW = TW + 2;  // branch tensor
  constexpr int PITCH = C * 2 + 16;
  constexpr int NS = C / 16, C8 = C / 8;
  __shared__ __attribute__((aligned(16))) unsigned char xp[XH * XW * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char tp[UH * UW * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lh = lane >> 5;
  int t = xcd_contiguous_tile(blockIdx.x, gridDim.x);
  const int tx = t % g.tiles_x;
  t /= g.tiles_x;
  const int ty = t % g.tiles_y;
  const int b = t / g.tiles_y;
  const int y0 = ty * TH, x0 = tx * TW;
  const uint16_t* img = g.x + (size_t)b * g.H * g.W * C;

  u32x4 wreg[9][NS];
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int s = 0; s < NS; ++s) wreg[tap][s] = g.wa[(tap * NS + s) * 64 + lane];

  stage_patch<C, PITCH, NT, XH, XW>(xp, img, g.H, g.W, y0 - 2, x0 - 2, true, tid);
  // Branch pixels outside the image are conv_b's zero padding; only the one-pixel ring of
  // the branch region can lie outside.
  if (y0 == 0 || x0 == 0 || y0 + TH >= g.H || x0 + TW >= g.W) {  // uniform: border tiles only
    constexpr int RING = 2 * UW + 2 * (UH - 2);
    for (int idx = tid; idx < RING * C8; idx += NT) {
      const int k = idx / C8, c8 = idx - k * C8;
      int py, px;
      if (k < UW) {
        py = 0; px = k;
      } else if (k < 2 * UW) {
        py = UH - 1; px = k - UW;
      } else {
        const int m = k - 2 * UW;
        py = 1 + (m >> 1); px = (m & 1) ? UW - 1 : 0;
      }
      const int y = y0 - 1 + py, x = x0 - 1 + px;
      if (y < 0 || y >= g.H || x < 0 || x >= g.W) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        *(u32x4*)(tp + (py * UW + px) * PITCH + c8 * 16) = z;
      }
    }
    // a ragged last tile also has interior rows / columns past the image
    if (y0 + TH > g.H || x0 + TW > g.W) {
      for (int idx = tid; idx < UH * UW * C8; idx += NT) {
        const int pix = idx / C8, c8 = idx - pix * C8;
        const int py = pix / UW, px = pix - py * UW;
        const int y = y0 - 1 + py, x = x0 - 1 + px;
        if (y >= g.H || x >= g.W) {
          const u32x4 z = {0u, 0u, 0u, 0u};
          *(u32x4*)(tp + pix * PITCH + c8 * 16) = z;
        }
      }
    }
  }
  __syncthreads();

  // the biases in the accumulator layout: register 4*q4 + u holds channel 8*q4 + 4*lh + u
  f32x16 ba_acc, bb_acc;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 av = *(const f32x4*)(g.ba + 8 * q4 + 4 * lh);
    const f32x4 bv = *(const f32x4*)(g.bb + 8 * q4 + 4 * lh);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ba_acc[4 * q4 + u] = av[u];
      bb_acc[4 * q4 + u] = bv[u];
    }
  }

  {  // conv_a over the in-image part of the branch region
    const int ur0 = y0 - 1, uc0 = x0 - 1;
    const int r_off = ur0 < 0 ? 1 : 0, c_off = uc0 < 0 ? 1 : 0;
    const int nrows = min(UH, g.H - ur0) - r_off, ncols = min(UW, g.W - uc0) - c_off;
    const int npix = nrows * ncols;
    const float inv_ncols = 1.0f / (float)ncols;
    for_wave_tiles<NW>(wave, npix, [&](auto cnt, int tile) {
      constexpr int N = decltype(cnt)::value;
      TilePixel px[N];
      const unsigned char* base[N];
      f32x16 acc[N];
#pragma unroll
      for (int n = 0; n < N; ++n) {
        px[n] = tile_pixel(tile + n * NW, li, npix, ncols, inv_ncols, r_off, c_off);
        base[n] = xp + (px[n].ry * XW + px[n].cx) * PITCH + lh * 16;
      }
      conv_taps<C, PITCH, N>(wreg, base, XW, ba_acc, acc);
#pragma unroll
      for (int n = 0; n < N; ++n) {
        if (!px[n].live) continue;
        unsigned char* dst = tp + (px[n].ry * UW + px[n].cx) * PITCH;
#pragma unroll
        for (int q4 = 0; q4 < C / 8; ++q4) {
          const int ch = 8 * q4 + 4 * lh;
          u32x2 ov;
          ov[0] = relu_h2(pack_f16(acc[n][4 * q4 + 0], acc[n][4 * q4 + 1]));
          ov[1] = relu_h2(pack_f16(acc[n][4 * q4 + 2], acc[n][4 * q4 + 3]));
          *(u32x2*)(dst + ch * 2) = ov;
        }
      }
    });
  }
  // conv_b's filter bank replaces conv_a's in the registers
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int s = 0; s < NS; ++s) wreg[tap][s] = g.wb[(tap * NS + s) * 64 + lane];
  __syncthreads();

  {
    const int nrows = min(TH, g.H - y0), ncols = min(TW, g.W - x0);
    const int npix = nrows * ncols;
    const float inv_ncols = 1.0f / (float)ncols;
    for_wave_tiles<NW>(wave, npix, [&](auto cnt, int tile) {
      constexpr int N = decltype(cnt)::value;
      TilePixel px[N];
      const unsigned char* base[N];
      size_t o[N];
      u32x2 xv[N][C / 8];
      f32x16 acc[N];
#pragma unroll
      for (int n = 0; n < N; ++n) {
        px[n] = tile_pixel(tile + n * NW, li, npix, ncols, inv_ncols, 0, 0);
        base[n] = tp + (px[n].ry * UW + px[n].cx) * PITCH + lh * 16;
        o[n] = ((size_t)(y0 + px[n].ry) * g.W + x0 + px[n].cx) * C;
#pragma unroll
        for (int q4 = 0; q4 < C / 8; ++q4) xv[n][q4] = *(const u32x2*)(img + o[n] + 8 * q4 + 4 * lh);
      }
      conv_taps<C, PITCH, N>(wreg, base, UW, bb_acc, acc);
      // (the residual is consumed outside the guard so that its load is not sunk behind
      // the MFMAs)
#pragma unroll
      for (int n = 0; n < N; ++n) {
        uint16_t* dst = g.out + (size_t)b * g.H * g.W * C + o[n];
#pragma unroll
        for (int q4 = 0; q4 < C / 8; ++q4) {
          const int ch = 8 * q4 + 4 * lh;
          float r[4];
          r[0] = acc[n][4 * q4 + 0] + f16_value(xv[n][q4][0] & 0xFFFFu);
          r[1] = acc[n][4 * q4 + 1] + f16_value(xv[n][q4][0] >> 16);
          r[2] = acc[n][4 * q4 + 2] + f16_value(xv[n][q4][1] & 0xFFFFu);
          r[3] = acc[n][4 * q4 + 3] + f16_value(xv[n][q4][1] >> 16);
          if (g.relu_out) {
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = fmaxf(r[u], 0.0f);
          }
          const u32x2 ov = {pack_f16(r[0], r[1]), pack_f16(r[2], r[3])};
          if (px[n].live) *(u32x2*)(dst + ch) = ov;
        }
      }
    });
  }
}

template <int CIN, int COUT, int PTH, int PTW>
hipError_t launch_pool_t(ConvPoolArgs g, hipStream_t st) {
  g.tiles_x = (g.Wo + PTW - 1) / PTW;
  g.tiles_y = (g.Ho + PTH - 1) / PTH;
  const long long blocks = (long long)g.B * g.tiles_x * g.tiles_y;
  conv3x3_pool_kernel<CIN, COUT, PTH, PTW, 4><<<(unsigned)blocks, 256, 0, st>>>(g);
  return hipGetLastError();
}

template <int CIN, int COUT>
hipError_t launch_pool_c(const ConvPoolArgs& g, hipStream_t st) {
  // Tile shapes are bounded by 64 KB of LDS per workgroup.  The byte-input convolution
  // (few MFMAs per pixel) takes six pooled rows per tile when that wastes little at the
  // bottom edge; the others ran faster with three (more workgroups per CU).
  if constexpr (CIN == 3 && COUT == 16) {
    const bool six = g.Ho % 6 == 0 || g.Ho > 18;
    if (g.Wo > 16)
      return six ? launch_pool_t<CIN, COUT, 6, 32>(g, st) : launch_pool_t<CIN, COUT, 3, 32>(g, st);
    return six ? launch_pool_t<CIN, COUT, 6, 16>(g, st) : launch_pool_t<CIN, COUT, 3, 16>(g, st);
  } else {
    return launch_pool_t<CIN, COUT, 3, 16>(g, st);
  }
}

template <int C, int TH, int TW>
hipError_t launch_block_t(BlockArgs g, hipStream_t st) {
  g.tiles_x = (g.W + TW - 1) / TW;
  g.tiles_y = (g.H + TH - 1) / TH;
  const long long blocks = (long long)g.B * g.tiles_x * g.tiles_y;
  res_block_kernel<C, TH, TW, 4><<<(unsigned)blocks, 256, 0, st>>>(g);
  return hipGetLastError();
}

}  // namespace

bool conv3x3_pool_supported(int cin, int cout, int W) {
  if (cin == 3) return (cout == 16 || cout == 32) && W % 4 == 0;
  return (cin == 16 || cin == 32) && (cout == 16 || cout == 32);
}

// in: planar bytes (cin == 3) or fp16 channels-last; wpk / bias32 as packed for the unfused
// stem / patch kernels with fp16 weights; out: fp16 [B][(H-1)/2+1][(W-1)/2+1][cout].
hipError_t launch_conv3x3_pool(const void* in, const uint16_t* wpk, const float* bias32, void* out,
                               int B, int H, int W, int cin, int cout, float obs_sub, float obs_mul,
                               hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  ConvPoolArgs g;
  g.in = in; g.wpk = (const u32x4*)wpk; g.bias = bias32; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.Ho = (H - 1) / 2 + 1; g.Wo = (W - 1) / 2 + 1;
  g.tiles_x = g.tiles_y = 0;
  g.obs_sub = obs_sub; g.obs_mul = obs_mul;
  if (cin == 3 && cout == 16) return launch_pool_c<3, 16>(g, st);
  if (cin == 3 && cout == 32) return launch_pool_c<3, 32>(g, st);
  if (cin == 16 && cout == 16) return launch_pool_c<16, 16>(g, st);
  if (cin == 16 && cout == 32) return launch_pool_c<16, 32>(g, st);
  if (cin == 32 && cout == 16) return launch_pool_c<32, 16>(g, st);
  if (cin == 32 && cout == 32) return launch_pool_c<32, 32>(g, st);
  return hipErrorInvalidValue;
}

bool res_block_supported(int c) { return c == 16 || c == 32; }

// x, out: fp16 [B][H][W][c], distinct buffers (tiles read their neighbours' x);
// wa / wb, ba / bb: the two convolutions as packed for the unfused patch kernel.
hipError_t launch_res_block(const void* x, const uint16_t* wa, const float* ba, const uint16_t* wb,
                            const float* bb, void* out, int B, int H, int W, int c, int relu_out,
                            hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  BlockArgs g;
  g.x = (const uint16_t*)x; g.wa = (const u32x4*)wa; g.wb = (const u32x4*)wb; g.ba = ba; g.bb = bb;
  g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W;
  g.tiles_x = g.tiles_y = 0;
  g.relu_out = relu_out;
  if (c == 16) {
    if (W <= 16) return launch_block_t<16, 9, 16>(g, st);
    return H % 12 == 0 ? launch_block_t<16, 12, 32>(g, st) : launch_block_t<16, 6, 32>(g, st);
  }
  if (c == 32) {
    if (W <= 16) return launch_block_t<32, 9, 16>(g, st);
    return launch_block_t<32, 6, 32>(g, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace sf

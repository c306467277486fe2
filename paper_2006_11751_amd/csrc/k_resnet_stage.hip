// All residual blocks of one stage of the residual encoder in one kernel, with the frame
// resident in LDS (the encoder follows IMPALA; paper, App. DMLab-30):
//   for every block:  x <- x + conv_b(relu(conv_a(relu(x)))),  3x3 / stride 1 / pad 1 convolutions,
// fp16 activations, 16-bit MFMA with fp32 accumulation.
//
// Run block by block on pixel tiles, every block reads its input from memory with a two-pixel
// halo, recomputes a one-pixel halo of the branch tensor and writes its output back: at the
// first stage's size (16 x 36 x 64 per frame, 8192 frames) that is 2.4 GB of traffic for two
// blocks and a quarter of the first convolution's work done twice.  Here a workgroup of eight
// waves owns a frame at a time: the residual stream x stays in registers (16-byte pieces, the
// thread that loaded a piece keeps it), relu(x) and the branch tensor stay in two LDS images
// with a ring of zero pixels around them (the convolutions' padding), and the frame crosses
// the memory bus once in each direction.  Per block:
//   conv_a: X = relu(x) -> T = relu(conv + bias)        (fp16, rounded as it is written)
//   conv_b: T -> X = conv + bias                         (fp16)
//   add:    x <- x + X (packed fp16), X <- relu(x) for the next block
// The next frame's pieces travel into registers meanwhile, and so does the next convolution's
// filter bank (two register sets in alternation).
//
// v_mfma_f32_32x32x16_f16: lane l supplies A[i = l%32][k = 8*(l/32) + e] and
// B[k = 8*(l/32) + e][j = l%32]; D[i][j] sits in lane j + 32*((i/4)%2), register
// (i%4) + 4*(i/8).  A = weights (i = output channel, rows >= C are zero), B = pixels: for filter
// tap (p, q) the B operand of pixel (y, x) is the 16-byte run of 8 channels at image pixel
// (y + p - 1, x + q - 1).  Frame width a power of two (64, 32 or 16): a 32-pixel tile is half a
// row, a row or two rows, and a tile's LDS addresses are a per-lane constant plus a term that
// is the same for all lanes.
#include <mutex>
#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kNW = 8;          // waves per workgroup
constexpr int kNT = 64 * kNW;
constexpr int kMaxConvs = 8;    // 2 * blocks per stage

__device__ inline unsigned pk_max0(unsigned w) {
  return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(f16x2, w), f16x2{0, 0}));
}
__device__ inline unsigned pk_add(unsigned a, unsigned b) {
  return __builtin_bit_cast(unsigned, __builtin_bit_cast(f16x2, a) + __builtin_bit_cast(f16x2, b));
}
__device__ inline unsigned pk_f16(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, f16x2));
}
__device__ inline u32x4 relu8(u32x4 v) {
  return u32x4{pk_max0(v[0]), pk_max0(v[1]), pk_max0(v[2]), pk_max0(v[3])};
}

// f(integral_constant<int, 0>), f(integral_constant<int, STEP>), ... below END
template <int STEP, class F, int... I>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I * STEP>{}), ...);
}
template <int END, int STEP, class F>
__device__ inline void static_for(F&& f) {
  static_for_impl<STEP>(f, std::make_integer_sequence<int, (END + STEP - 1) / STEP>{});
}

struct StageArgs {
  const u32x4* x;              // fp16 [B][H][W][C] as 16-byte pieces
  u32x4* out;                  // the same shape
  const u32x4* w[kMaxConvs];   // A operands of conv_a, conv_b of every block: [9][C/16][64], or
                               // [5][64] tap pairs for 16 channels (res_stage_pack16)
  const float* bias[kMaxConvs];  // [32] each
  int B, H, n_convs, relu_out;
  int F;  // frames stacked into one LDS image (32 channels; 1 otherwise)
};

// C channels (16 or 32), frame width 1 << LW, PPT 16-byte pieces of a frame per thread; RES: the
// filter banks of all (at most four) convolutions stay in registers (16 channels only).
template <int C, int LW, int PPT, bool RES>
__global__ __launch_bounds__(kNT, 1) void res_stage_kernel(StageArgs g) {
  constexpr int W = 1 << LW;
  constexpr int C8 = C / 8, NS = C / 16;
  // Pixel pitch: 64 + 16 bytes for 32 channels, 32 bytes for 16 channels (a pitch of 48 would
  // not leave room for two images of the benchmark's first stage).  Measured on gfx950 with all
  // 16 waves of a CU reading: a 16-byte-per-lane read takes 4 cycles when the lanes' addresses
  // are 16, 48 or 80 bytes apart, 8 at 32 and 16 at 64 (bank conflicts).  At pitch 32 the two
  // 16-byte halves of a pixel are therefore swapped in every second group of eight pixels (bit
  // 3 of the pixel's column): reads are back at 4 cycles and the 8-byte accumulator stores take
  // 8 cycles instead of 16.
  constexpr int PITCH = C == 16 ? 32 : 80;
  constexpr bool SWZ = C == 16;
  auto swz = [](int col) { return SWZ ? ((col >> 3) & 1) << 4 : 0; };
  constexpr int ROW = (W + 2) * PITCH;  // image row pitch in bytes, ring included
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (scalar: tile loops branch uniformly)
  const int li = lane & 31, lh = lane >> 5;
  // Small frames (the 9 x 16 frames of the benchmark's last stage are 4.5 tiles for 8 waves) are
  // stacked F to an LDS image, one zero row between two frames: that row is the padding of both,
  // the convolutions run over the stack as over one tall frame and store nothing into the
  // separating rows, and the pieces of the F frames (contiguous in memory) skip them.
  const int frame_pieces = g.H * W * C8;
  const int HS = g.F * (g.H + 1) - 1;  // rows of the stack
  const int npix = HS * W;
  const int pieces = g.F * frame_pieces;  // of a full stack
  const int n_groups = (g.B + g.F - 1) / g.F;
  const int n_tiles = (npix + 31) >> 5;
  // image rows: the frame, the ring, and the rows that the lanes of a partial last tile look at
  // (zeros, like the ring; those lanes store nothing)
  const int img_bytes = (((n_tiles << 5) + W - 1) / W + 2) * ROW;
  unsigned char* X = lds;
  unsigned char* T = lds + img_bytes;
  float* bias_lds = (float*)(lds + 2 * img_bytes);  // [n_convs][32]: a convolution's first MFMA
                                                    // must not wait for a load from memory

  // both images start as zeros: the ring is never written again
  for (int i = tid; i < 2 * img_bytes / 16; i += kNT) ((u32x4*)lds)[i] = u32x4{0u, 0u, 0u, 0u};
  for (int i = tid; i < g.n_convs * 32; i += kNT) bias_lds[i] = g.bias[i >> 5][i & 31];

  // this thread's pieces: LDS byte offset of piece tid + k * kNT (past the end: piece 0, unused)
  // (shifts and masks: computed where it is used rather than kept in registers)
  auto poff = [&](int k) {
    const int p = tid + k * kNT;
    const int pc = p < pieces ? p : 0;
    const int pix = pc / C8, c8 = pc - pix * C8;
    const int ya = pix >> LW, x = pix & (W - 1);
    // row within the stack: one separating row per frame before it (F <= 4)
    const int y = ya + (ya >= g.H) + (ya >= 2 * g.H) + (ya >= 3 * g.H);
    return ((y + 1) * (W + 2) + x + 1) * PITCH + ((c8 * 16) ^ swz(x + 1));
  };
  // pieces of stack b that exist (the last stack may hold fewer frames)
  auto valid_pieces = [&](int b) { return min(g.F, g.B - b * g.F) * frame_pieces; };
  // this lane's pixel of tile 0 (for W >= 32 a tile lies in one row and the others follow by a
  // uniform step; for W = 16 a tile is two rows): byte offset of image pixel (y, x) of the
  // ring-less frame = ring pixel (y, x), i.e. the window origin of tap (0, 0)
  const int lane_row = (li >> LW) * ROW, lane_col = li & (W - 1);
  // fragment of filter column q: ring column lane_col + q (tile columns start at multiples of
  // 16, so the swizzle bit is that of lane_col + q); accumulator store of channel quad q4:
  // ring column lane_col + 1
  int lane_q[3], lane_o[C8];
#pragma unroll
  for (int q = 0; q < 3; ++q) lane_q[q] = lane_row + (lane_col + q) * PITCH + ((lh * 16) ^ swz(lane_col + q));
#pragma unroll
  for (int q4 = 0; q4 < C8; ++q4)
    lane_o[q4] = lane_row + ROW + (lane_col + 1) * PITCH + (((q4 * 16) ^ swz(lane_col + 1)) + lh * 8);

  u32x4 xs[PPT], nx[PPT];
  auto load_frame = [&](int b, u32x4 (&dst)[PPT]) {
    const u32x4* src = g.x + (size_t)b * pieces;
    const int valid = valid_pieces(b);
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      // (an opaque move keeps the index from being computed ahead of the frame loop, where it
      // would be spilled: its reload would wait for the previous frame's stores to complete)
      int p = tid;
      asm volatile("" : "+v"(p));
      p += k * kNT;
      dst[k] = src[p < valid ? p : valid - 1];
    }
  };
  // A operands of a convolution: nine taps x NS channel groups for the 32x32x16 MFMA; five tap
  // pairs for the 16x16x32 MFMA that runs the 16-channel stages (see conv16 below)
  constexpr bool M16 = C == 16;
  constexpr int NB = M16 ? 5 : 9;
  u32x4 wA[NB][NS], wB[NB][NS];
  auto load_bank = [&](int k, u32x4 (&dst)[NB][NS]) {
    const u32x4* src = g.w[k];
#pragma unroll
    for (int tap = 0; tap < NB; ++tap)
#pragma unroll
      for (int s = 0; s < NS; ++s) dst[tap][s] = src[(tap * NS + s) * 64 + lane];
  };
  // the bias of convolution k in the accumulator layout: register 4*q4 + u holds channel
  // 8*q4 + 4*lh + u
  auto bias_acc = [&](int k) {
    f32x16 a;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 bv = *(const f32x4*)(bias_lds + 32 * k + 8 * q4 + 4 * lh);
#pragma unroll
      for (int u = 0; u < 4; ++u) a[4 * q4 + u] = bv[u];
    }
    return a;
  };

  // One convolution over the frame: the wave's tiles wave, wave + 8, ... two at a time (two
  // independent MFMA chains), from image `src` into image `dst`.
  auto conv32 = [&](const u32x4 (&wreg)[NB][NS], int kconv, const unsigned char* src, unsigned char* dst,
                    bool relu) {
    const f32x16 init = bias_acc(kconv);
    auto tile_off = [&](int t) {  // byte offset of the tile's first pixel row / half row
      if (LW >= 5) return ((t << 5) >> LW) * ROW + ((t << 5) & (W - 1)) * PITCH;
      return (t * (32 >> LW)) * ROW;
    };
    auto run = [&](auto cnt, int t0) {
      constexpr int N = decltype(cnt)::value;
      f32x16 acc[N];
      const unsigned char* base[N];
#pragma unroll
      for (int n = 0; n < N; ++n) {
        acc[n] = init;
        base[n] = src + tile_off(t0 + n * kNW);
      }
      // K steps (tap, 16-channel group) in order; the pixel fragment of step k + D is requested
      // right behind the MFMA of step k (D register sets per tile), so that an LDS read has
      // D * N MFMAs to come back in.  (Left alone, the scheduler sinks each read to its use.)
      // One 16-byte read per MFMA is what bounds this loop: the four SIMDs of a CU share the
      // LDS, which measured 16 cycles per such read against 32 cycles per MFMA.  (Sharing one
      // read among a filter row's three taps by moving fragments down one lane with DPP, the
      // last lane of each 16-lane row fetching its own pixel, was tried: correct, but the moves,
      // the masked reads and 30 more registers made the kernel 25 % slower.)
      constexpr int S = 9 * NS;
      auto frag_off = [&](int k) {
        const int tap = k / NS, sg = k - tap * NS;
        return lane_q[tap % 3] + (tap / 3) * ROW + sg * 32;
      };
      // (D register sets: two, or one where nine pieces per thread leave no room for the second)
      constexpr int D = PPT >= 9 ? 1 : 2;
      u32x4 pf[D][N];
#pragma unroll
      for (int n = 0; n < N; ++n)
#pragma unroll
        for (int d = 0; d < D; ++d) pf[d][n] = *(const u32x4*)(base[n] + frag_off(d));
#pragma unroll
      for (int k = 0; k < S; ++k) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
          acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, wreg[k / NS][k % NS]),
                                                          __builtin_bit_cast(f16x8, pf[k % D][n]), acc[n], 0, 0, 0);
          if (k + D < S) pf[k % D][n] = *(const u32x4*)(base[n] + frag_off(k + D));
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int n = 0; n < N; ++n) {
        const int t = t0 + n * kNW;
        if ((t << 5) + li >= npix) continue;  // (a last tile may be partial)
        if (g.F > 1) {  // (a row between two stacked frames stays zero)
          const int ys = ((t << 5) + li) >> LW;
          if (ys == g.H || ys == 2 * g.H + 1 || ys == 3 * g.H + 2) continue;
        }
        // the lane's pixel in dst: ring pixel (y + 1, x + 1)
        unsigned char* o = dst + tile_off(t);
#pragma unroll
        for (int q4 = 0; q4 < C8; ++q4) {
          u32x2 ov;
          ov[0] = pk_f16(acc[n][4 * q4 + 0], acc[n][4 * q4 + 1]);
          ov[1] = pk_f16(acc[n][4 * q4 + 2], acc[n][4 * q4 + 3]);
          if (relu) {
            ov[0] = pk_max0(ov[0]);
            ov[1] = pk_max0(ov[1]);
          }
          *(u32x2*)(o + lane_o[q4]) = ov;
        }
      }
    };
    // (32 channels with five or more pieces per thread: two filter banks of 72 registers and
    // the frame's pieces leave no room for a second tile's accumulators; spills would go to
    // memory, 260 MB per launch at the benchmark's second stage)
    constexpr bool kPairs = !(C == 32 && PPT >= 5);
    if constexpr (!M16) {  // (the tile code is instantiated for 32 channels only)
      int t = wave;
      if (kPairs)
        for (; t + kNW < n_tiles; t += 2 * kNW) run(std::integral_constant<int, 2>{}, t);
      for (; t < n_tiles; t += kNW) run(std::integral_constant<int, 1>{}, t);
    }
  };

  // The same for 16 channels on v_mfma_f32_16x16x32_f16 (a 32x32 tile would compute 16 output
  // rows of zeros): lane l supplies A[i = l%16][k = 8*(l/16) + e] and B[k][j = l%16]; D[i][j] sits
  // in lane j + 16*(i/4), register i%4.  A tile is 16 neighbouring pixels of a row; K = 32 is two
  // filter taps x 16 channels, lane group g = l/16 holding tap g%2 of the pair, channels
  // 8*(g/2)..: with the two taps side by side in a filter row, the 64 lanes' 16-byte reads are
  // free of bank conflicts (4 cycles measured; 8 with the channel half in the low bit of g, and 8
  // for two taps of different rows).  Five MFMAs: taps (0,1), (3,4), (6,7), (2,5), (8, none: zero
  // weights, the lanes re-read tap 8).
  const int j16 = lane & 15, g16 = lane >> 4;
  int lane_m[5], lane_o16;
  {
    constexpr int pair[5][2] = {{0, 1}, {3, 4}, {6, 7}, {2, 5}, {8, 8}};
#pragma unroll
    for (int m = 0; m < 5; ++m) {
      const int tap = pair[m][g16 & 1], p = tap / 3, q = tap % 3;
      lane_m[m] = p * ROW + (j16 + q) * PITCH + (((g16 >> 1) * 16) ^ swz(j16 + q));
    }
    // channels 4*g .. 4*g+3 of ring pixel (y + 1, x + 1)
    lane_o16 = ROW + (j16 + 1) * PITCH + ((((g16 >> 1) * 16) ^ swz(j16 + 1)) + (g16 & 1) * 8);
  }
  auto conv16 = [&](const u32x4 (&wreg)[NB][NS], int kconv, const unsigned char* src, unsigned char* dst,
                    bool relu) {
    const f32x4 init = *(const f32x4*)(bias_lds + 32 * kconv + 4 * g16);
    const int n16 = npix >> 4;  // (the width is a multiple of 16: no partial tiles)
    auto tile_off = [&](int t) { return ((t << 4) >> LW) * ROW + ((t << 4) & (W - 1)) * PITCH; };
    auto run = [&](auto cnt, int t0) {
      constexpr int N = decltype(cnt)::value;
      f32x4 acc[N];
      const unsigned char* base[N];
#pragma unroll
      for (int n = 0; n < N; ++n) {
        acc[n] = init;
        base[n] = src + tile_off(t0 + n * kNW);
      }
      // the pixel fragment of step k + 2 is requested right behind the MFMA of step k
      u32x4 pf[2][N];
#pragma unroll
      for (int n = 0; n < N; ++n)
#pragma unroll
        for (int d = 0; d < 2; ++d) pf[d][n] = *(const u32x4*)(base[n] + lane_m[d]);
#pragma unroll
      for (int k = 0; k < 5; ++k) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, wreg[k][0]),
                                                          __builtin_bit_cast(f16x8, pf[k & 1][n]), acc[n], 0, 0, 0);
          if (k + 2 < 5) pf[k & 1][n] = *(const u32x4*)(base[n] + lane_m[k + 2]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int n = 0; n < N; ++n) {
        u32x2 ov;
        ov[0] = pk_f16(acc[n][0], acc[n][1]);
        ov[1] = pk_f16(acc[n][2], acc[n][3]);
        if (relu) {
          ov[0] = pk_max0(ov[0]);
          ov[1] = pk_max0(ov[1]);
        }
        *(u32x2*)(dst + tile_off(t0 + n * kNW) + lane_o16) = ov;
      }
    };
    if constexpr (M16) {
      int t = wave;
      // (four tiles in flight, two where the resident filter banks leave no room for more)
      if constexpr (!(RES && PPT >= 9))
        for (; t + 3 * kNW < n16; t += 4 * kNW) run(std::integral_constant<int, 4>{}, t);
      for (; t + kNW < n16; t += 2 * kNW) run(std::integral_constant<int, 2>{}, t);
      for (; t < n16; t += kNW) run(std::integral_constant<int, 1>{}, t);
    }
  };
  auto conv = [&](const u32x4 (&wreg)[NB][NS], int kconv, const unsigned char* src, unsigned char* dst,
                  bool relu) {
    if constexpr (M16) conv16(wreg, kconv, src, dst, relu);
    else conv32(wreg, kconv, src, dst, relu);
  };

  if constexpr (M16) {
    // 16 channels: the residual stream lives in the accumulator layout of the wave that owns the
    // tile (lane j + 16*g: channels 4g..4g+3 of pixel j, 8 bytes; tiles wave, wave + 8, ...), so
    // conv_b's epilogue adds it in registers and writes relu(x) for the next block straight into
    // X: no separate pass over the frame, one barrier fewer per block.  Same arithmetic as the
    // piece form: conv_b's result is rounded to fp16, then added to x in fp16.
    constexpr int RT = 2 * PPT;  // 16-pixel tiles per wave at most
    const int n16 = npix >> 4;
    u32x2 xt[RT], nt[RT];
    auto tile_off16 = [&](int t) { return ((t << 4) >> LW) * ROW + ((t << 4) & (W - 1)) * PITCH; };
    const int lane_g = j16 * 32 + g16 * 8;  // the lane's 8 bytes within a tile's 512 in memory
    // (part p of `parts`: rounds p, p + parts, ...)
    auto load_tiles = [&](int bb, u32x2 (&dst)[RT], int part = 0, int parts = 1) {
      const unsigned char* src = (const unsigned char*)g.x + (size_t)bb * pieces * 16;
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        if (r % parts != part) continue;
        // (an opaque move keeps the offsets from being computed ahead of the frame loop and spilled)
        int o = lane_g;
        asm volatile("" : "+v"(o));
        const int t = wave + kNW * r;
        dst[r] = *(const u32x2*)(src + (size_t)(t < n16 ? t : n16 - 1) * 512 + o);
      }
    };
    auto relu2 = [](u32x2 v) { return u32x2{pk_max0(v[0]), pk_max0(v[1])}; };
    // conv_b of a block: T -> x += conv + bias; X <- relu(x) if another block follows.  The tile
    // rounds are unrolled (the stream's registers are indexed by the round).
    auto conv16_b = [&](const u32x4 (&wreg)[NB][NS], int kconv, bool more) {
      const f32x4 init = *(const f32x4*)(bias_lds + 32 * kconv + 4 * g16);
      auto run = [&](auto cnt, auto r0c) {
        constexpr int N = decltype(cnt)::value, R0 = decltype(r0c)::value;
        f32x4 acc[N];
        const unsigned char* base[N];
#pragma unroll
        for (int n = 0; n < N; ++n) {
          acc[n] = init;
          base[n] = T + tile_off16(wave + kNW * (R0 + n));
        }
        u32x4 pf[2][N];
#pragma unroll
        for (int n = 0; n < N; ++n)
#pragma unroll
          for (int d = 0; d < 2; ++d) pf[d][n] = *(const u32x4*)(base[n] + lane_m[d]);
#pragma unroll
        for (int k = 0; k < 5; ++k) {
#pragma unroll
          for (int n = 0; n < N; ++n) {
            acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, wreg[k][0]),
                                                            __builtin_bit_cast(f16x8, pf[k & 1][n]), acc[n], 0, 0, 0);
            if (k + 2 < 5) pf[k & 1][n] = *(const u32x4*)(base[n] + lane_m[k + 2]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
        for (int n = 0; n < N; ++n) {
          if (R0 + n < RT) {  // (constant once unrolled)
            u32x2& x = xt[R0 + n < RT ? R0 + n : RT - 1];
            x[0] = pk_add(x[0], pk_f16(acc[n][0], acc[n][1]));
            x[1] = pk_add(x[1], pk_f16(acc[n][2], acc[n][3]));
            if (more) *(u32x2*)(X + tile_off16(wave + kNW * (R0 + n)) + lane_o16) = relu2(x);
          }
        }
      };
      if constexpr (RES && PPT >= 9) {
        static_for<RT, 2>([&](auto r0c) {
          constexpr int R0 = decltype(r0c)::value;
          const int t0 = wave + kNW * R0;
          if (t0 + kNW < n16 && R0 + 1 < RT) run(std::integral_constant<int, 2>{}, r0c);
          else if (t0 < n16) run(std::integral_constant<int, 1>{}, r0c);
        });
      } else {
        static_for<RT, 4>([&](auto r0c) {
          constexpr int R0 = decltype(r0c)::value;
          const int t0 = wave + kNW * R0;
          if (t0 + 3 * kNW < n16 && R0 + 3 < RT) {
            run(std::integral_constant<int, 4>{}, r0c);
          } else if (t0 < n16) {
            if (t0 + kNW < n16 && R0 + 1 < RT) {
              run(std::integral_constant<int, 2>{}, r0c);
              if (t0 + 2 * kNW < n16 && R0 + 2 < RT) run(std::integral_constant<int, 1>{}, std::integral_constant<int, R0 + 2>{});
            } else {
              run(std::integral_constant<int, 1>{}, r0c);
            }
          }
        });
      }
    };

    int b = blockIdx.x;
    load_tiles(b, xt);
    // Up to two blocks: all four filter banks stay in registers (80), so that the next frame's
    // tiles are the only loads in flight while a frame is computed.  The load counter completes in
    // order: a filter bank requested behind the frame's 18 loads per lane would arrive only after
    // them, and a wait for a bank requested ahead of them is sized by the compiler for the loop's
    // other trips, where fewer loads follow it, so that it caught 14 of the 18 (14 k of a frame's
    // 42 k cycles, measured with cycle stamps).
    constexpr bool resident = RES;
    u32x4 wk[RES ? 4 : 1][NB][NS];
    if constexpr (resident) {
#pragma unroll
      for (int c = 0; c < 4; ++c) load_bank(c < g.n_convs ? c : 0, wk[c]);
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the banks (and the first frame) have arrived
    } else {
      load_bank(0, wA);
    }
    __syncthreads();  // zeros in place
    for (; b < g.B; b += gridDim.x) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        const int t = wave + kNW * r;
        if (t < n16) *(u32x2*)(X + tile_off16(t) + lane_o16) = relu2(xt[r]);
      }
      __syncthreads();
      const int bn = b + (int)gridDim.x < g.B ? b + (int)gridDim.x : b;  // (last round: its own again)
      if constexpr (resident) {
        // the next frame is requested in three parts between the convolutions: the requests of
        // all workgroups in one burst kept the last waves of a workgroup 10 k cycles at issuing theirs
        load_tiles(bn, nt, 0, 3);
        conv16(wk[0], 0, X, T, true);
        load_tiles(bn, nt, 1, 3);
        __syncthreads();
        conv16_b(wk[1], 1, g.n_convs > 2);
        load_tiles(bn, nt, 2, 3);
        __syncthreads();  // X complete for the next block / T free for the next frame
        if (g.n_convs > 2) {
          conv16(wk[2], 2, X, T, true);
          __syncthreads();
          conv16_b(wk[3], 3, false);
          __syncthreads();
        }
      } else {
        load_tiles(bn, nt);
        for (int k = 0; k < g.n_convs; k += 2) {
          load_bank(k + 1, wB);
          conv16(wA, k, X, T, true);
          __syncthreads();
          load_bank(k + 2 < g.n_convs ? k + 2 : 0, wA);
          conv16_b(wB, k + 1, k + 2 < g.n_convs);
          __syncthreads();
        }
      }
      unsigned char* dst = (unsigned char*)g.out + (size_t)b * pieces * 16;
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        int o = lane_g;
        asm volatile("" : "+v"(o));
        const int t = wave + kNW * r;
        if (t < n16) *(u32x2*)(dst + (size_t)t * 512 + o) = g.relu_out ? relu2(xt[r]) : xt[r];
      }
#pragma unroll
      for (int r = 0; r < RT; ++r) xt[r] = nt[r];
    }
    return;
  }

  int b = blockIdx.x;
  load_frame(b, xs);
  load_bank(0, wA);
  __syncthreads();  // zeros in place
  for (; b < n_groups; b += gridDim.x) {
#pragma unroll
    for (int k = 0; k < PPT; ++k)
      if (tid + k * kNT < pieces) *(u32x4*)(X + poff(k)) = relu8(xs[k]);
    __syncthreads();
    load_frame(b + (int)gridDim.x < n_groups ? b + (int)gridDim.x : b, nx);  // (last round: its own again)
    for (int k = 0; k < g.n_convs; k += 2) {
      // conv_a of the block: X -> T, ReLU; conv_b's bank arrives meanwhile
      load_bank(k + 1, wB);
      conv(wA, k, X, T, true);
      __syncthreads();
      // conv_b: T -> X; the next conv_a's bank (the next block's, or the first of the next frame)
      load_bank(k + 2 < g.n_convs ? k + 2 : 0, wA);
      conv(wB, k + 1, T, X, false);
      __syncthreads();
      // x <- x + branch; X <- relu(x) unless this was the last block.  Three pieces at a time:
      // their reads first, then the arithmetic and the writes (one LDS latency per three pieces).
      const bool more = k + 2 < g.n_convs;
#pragma unroll
      for (int k0 = 0; k0 < PPT; k0 += 3) {
        u32x4 u[3];
#pragma unroll
        for (int j = 0; j < 3; ++j)
          if (k0 + j < PPT) u[j] = *(const u32x4*)(X + poff(k0 + j));
#pragma unroll
        for (int j = 0; j < 3; ++j)
          if (k0 + j < PPT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) xs[k0 + j][e] = pk_add(xs[k0 + j][e], u[j][e]);
            if (more && tid + (k0 + j) * kNT < pieces) *(u32x4*)(X + poff(k0 + j)) = relu8(xs[k0 + j]);
          }
      }
      if (more) __syncthreads();
    }
    // (the piece index goes through an opaque move: offsets computed ahead of the loop would be
    // spilled, and a reload between two stores waits for the first store to complete)
    u32x4* dst = g.out + (size_t)b * pieces;
    const int valid = valid_pieces(b);
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      int p = tid;
      asm volatile("" : "+v"(p));
      p += k * kNT;
      if (p < valid) dst[p] = g.relu_out ? relu8(xs[k]) : xs[k];
    }
#pragma unroll
    for (int k = 0; k < PPT; ++k) xs[k] = nx[k];
  }
}

// (H: rows of the stack)
size_t stage_lds_bytes(int c, int H, int W) {
  const int pitch = c == 16 ? 32 : 80;
  const int n_tiles = (H * W + 31) / 32;
  const int rows = (n_tiles * 32 + W - 1) / W + 2;  // as in the kernel
  return 2 * (size_t)rows * (W + 2) * pitch + kMaxConvs * 32 * sizeof(float);  // + the biases
}

template <int C, int LW, int PPT, bool RES>
hipError_t launch_stage_r(const StageArgs& g, size_t lds, hipStream_t st) {
  auto kern = res_stage_kernel<C, LW, PPT, RES>;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&] {
    attr_status = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  if (attr_status != hipSuccess) return attr_status;
  // one workgroup per CU, each walking its share of the frames
  const int groups = (g.B + g.F - 1) / g.F;
  const int blocks = groups < 256 ? groups : 256;
  kern<<<blocks, kNT, lds, st>>>(g);
  return hipGetLastError();
}

template <int C, int LW, int PPT>
hipError_t launch_stage_t(const StageArgs& g, size_t lds, hipStream_t st) {
  if constexpr (C == 16) {
    if (g.n_convs <= 4) return launch_stage_r<C, LW, PPT, true>(g, lds, st);
  }
  return launch_stage_r<C, LW, PPT, false>(g, lds, st);
}

}  // namespace

// A operands of a 16 -> 16 channel convolution for the tap-pair MFMAs of the stage kernel:
// wpk[(m * 64 + lane) * 8 + e] = w[n = lane%16][c = 8*(lane/32) + e][tap], tap = pair m's first
// (lane/16 even) or second (odd) member; pair 4 has no second member (zeros).
void res_stage_pack16(const float* w, bool f16, std::vector<uint16_t>& wpk) {
  static const int pair[5][2] = {{0, 1}, {3, 4}, {6, 7}, {2, 5}, {8, -1}};
  wpk.assign((size_t)5 * 64 * 8, 0);
  for (int m = 0; m < 5; ++m)
    for (int lane = 0; lane < 64; ++lane)
      for (int e = 0; e < 8; ++e) {
        const int n = lane & 15, grp = lane >> 4, c = 8 * (grp >> 1) + e, tap = pair[m][grp & 1];
        if (tap >= 0)
          wpk[((size_t)m * 64 + lane) * 8 + e] =
              conv_weight_bits(w[(((size_t)n * 16 + c) * 3 + tap / 3) * 3 + tap % 3], f16);
      }
}

// Shapes: 16 or 32 channels, frame width 16, 32 or 64, both LDS images within 160 KB, at most
// nine 16-byte pieces per thread, one to four blocks; and at least one 32-pixel tile per wave,
// for which 32-channel frames smaller than that are stacked two to four to an image.
namespace {
// Frames per LDS image: 1 where a frame has a tile for every wave; else (32 channels) the
// stack of 2 to 4 frames that fills the waves' tile rounds best; 0: not a shape for this kernel.
int stage_frames(int c, int H, int W) {
  if ((c != 16 && c != 32) || (W != 16 && W != 32 && W != 64) || H < 1) return 0;
  auto fits = [&](int F) {
    const int HS = F * (H + 1) - 1;
    return stage_lds_bytes(c, HS, W) <= 160 * 1024 && (F * H * W * c / 8 + kNT - 1) / kNT <= 9;
  };
  if ((H * W + 31) / 32 >= kNW) return fits(1) ? 1 : 0;
  if (c != 32) return 0;
  int best = 0;
  double best_fill = 0.0;
  for (int F = 2; F <= 4; ++F) {
    const int tiles = ((F * (H + 1) - 1) * W + 31) / 32;
    if (tiles < kNW || !fits(F)) continue;
    // useful pixels per tile slot of the rounds the waves go through
    const double fill = (double)F * H * W / (32.0 * kNW * ((tiles + kNW - 1) / kNW));
    if (fill > best_fill) {
      best_fill = fill;
      best = F;
    }
  }
  return best;
}
}  // namespace

bool res_stage_supported(int c, int H, int W, int n_blocks) {
  if (n_blocks < 1 || 2 * n_blocks > kMaxConvs) return false;
  return stage_frames(c, H, W) > 0;
}

// x, out: fp16 [B][H][W][c] (may be the same buffer: a workgroup reads a frame before it
// writes it, and frames are not shared); wpk[k], bias[k]: the stage's block convolutions in
// order (conv_a, conv_b of block 1, ...), packed as for the patch kernels with fp16 weights.
hipError_t launch_res_stage(const void* x, void* out, const uint16_t* const* wpk, const float* const* bias,
                            int n_convs, int B, int H, int W, int c, int relu_out, hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  if (!res_stage_supported(c, H, W, n_convs / 2) || (n_convs & 1)) return hipErrorInvalidValue;
  StageArgs g;
  g.x = (const u32x4*)x; g.out = (u32x4*)out;
  for (int k = 0; k < kMaxConvs; ++k) {
    g.w[k] = (const u32x4*)wpk[k < n_convs ? k : 0];
    g.bias[k] = bias[k < n_convs ? k : 0];
  }
  g.B = B; g.H = H; g.n_convs = n_convs; g.relu_out = relu_out;
  g.F = stage_frames(c, H, W);
  const size_t lds = stage_lds_bytes(c, g.F * (H + 1) - 1, W);
  const int ppt = (g.F * H * W * c / 8 + kNT - 1) / kNT;
#define SF_STAGE(C, LW)                                                    \
  do {                                                                     \
    if (ppt <= 2) return launch_stage_t<C, LW, 2>(g, lds, st);             \
    if (ppt <= 5) return launch_stage_t<C, LW, 5>(g, lds, st);             \
    return launch_stage_t<C, LW, 9>(g, lds, st);                           \
  } while (0)
  if (c == 16) {
    if (W == 64) SF_STAGE(16, 6);
    if (W == 32) SF_STAGE(16, 5);
    SF_STAGE(16, 4);
  }
  if (W == 64) SF_STAGE(32, 6);
  if (W == 32) SF_STAGE(32, 5);
  SF_STAGE(32, 4);
#undef SF_STAGE
}

}  // namespace sf

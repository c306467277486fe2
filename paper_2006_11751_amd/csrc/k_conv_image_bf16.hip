// Strided convolution of the plain encoder in bf16 configurations with the frame's whole
// input image resident in LDS (paper, App. "Model architectures": conv layers behind the
// first one), 16-bit MFMA with fp32 accumulation, bf16 activations in and out.
//
//   out[b][oy][ox][n] = act(bias[n] + sum_{p,q,c} in[b][oy*s + p][ox*s + q][c] * W[n][c][p][q])
//
// The tiled implicit-GEMM kernel is bound by the bytes it moves from L2 into LDS: an input
// pixel of a 4x4 / stride 2 layer is staged four times (once per filter window that covers it)
// and every K chunk costs a barrier.  Here a workgroup owns one frame: its channels-last image
// (17 x 31 pixels x 64 bytes for the standard network) is copied into LDS once, and after one
// barrier each wave runs the whole K loop without further synchronisation: pixel fragments
// straight from the image at the filter tap's offset, weight fragments (packed per lane) out
// of registers, where the wave's whole filter bank stays while the workgroup walks its frames;
// the next frame's image travels into registers while the current one is computed.
//
// v_mfma_f32_16x16x32_bf16: lane l supplies A[i = l%16][k = 8*(l/16) + e] and
// B[k = 8*(l/16) + e][j = l%16], e = 0..7 (16 bytes each); D[i][j] sits in lane j + 16*(i/4),
// register i%4.  A = weights (i = output channel), B = pixels, so a lane ends up with four
// consecutive channels of one pixel (one 8-byte store).  One instruction covers one filter tap
// (32 input channels).  Wave w owns output channels 16w .. 16w+15 of the workgroup's 64 and all
// MT 16-pixel tiles of the frame: each weight fragment feeds MT independent MFMAs.
//
// LDS layout: pixel pitch 64 + 16 bytes = 5 pieces of 16 bytes, rows padded so that output
// pixel n of the frame (row-major) reads piece 10 * n + const modulo 16 also across the end of
// an output row.  A 16-byte LDS read serves eight lanes per pass, lanes 4j .. 4j+3 together
// with lanes 4(j^1) + 16 .. +3; with the four lane groups one piece apart and neighbouring
// pixels 10 pieces apart every pass touches eight different pieces.
#include <string.h>

#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr size_t kMaxLds = 64 * 1024;  // the default dynamic LDS limit; two workgroups per CU

struct ImageArgs {
  const u32x4* in;    // bf16 [B][H][W][32], 4 pieces per pixel
  const u32x4* wpk;   // [N/16][KS*KS][64] lane fragments
  const float* bias;  // [N]
  uint16_t* out;      // bf16 [B][Ho*Wo][N]
  int B, H, W, Ho, Wo, N, relu;
  int row_pad;        // 16-byte pieces appended to every image row in LDS
};

template <int KS, int STRIDE, int MT>
__global__ __launch_bounds__(256, 2) void conv_image_bf16_kernel(ImageArgs g) {
  constexpr int C4 = 4;        // 16-byte pieces per pixel (32 channels)
  constexpr int P4 = C4 + 1;   // LDS pixel pitch in pieces
  constexpr int G = KS * KS;   // K groups = filter taps
  constexpr int NV = 9;        // image pieces per thread: 17 x 31 pixels x 4 = 2108 <= 9 * 256
  extern __shared__ __attribute__((aligned(16))) u32x4 img[];  // [H][row_stride] pieces

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lp = lane & 15, lg = lane >> 4;
  const int ntile = blockIdx.y * 4 + wave;  // 16 output channels
  const int npix_in = g.H * g.W, npix_out = g.Ho * g.Wo;
  const int row_stride = g.W * P4 + g.row_pad;
  const int total = npix_in * C4;

  // The wave's whole filter bank (16 channels x 16 taps x 32 input channels) stays in
  // registers for all frames of the workgroup.
  u32x4 wf[G];
#pragma unroll
  for (int t = 0; t < G; ++t) wf[t] = g.wpk[((size_t)ntile * G + t) * 64 + lane];
  const f32x4 bias4 = *(const f32x4*)(g.bias + ntile * 16 + 4 * lg);

  // this thread's pieces of a frame image: source index and LDS index
  auto piece = [&](int u) {  // past the end: the last piece again (same bits, same place)
    const int f = tid + 256 * u;
    return f < total ? f : total - 1;
  };
  int lds_idx[NV];
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int f = piece(u);
    const int pix = f >> 2, c4 = f & 3;
    const int y = pix / g.W, x = pix - y * g.W;
    lds_idx[u] = y * row_stride + x * P4 + c4;
  }
  // this lane's pixel of every tile: LDS index of its window's first pixel plus the lane
  // group's channel piece, and its output offset.  Pixels past the end repeat the last one
  // (computed again, stored again with the same bits: no per-lane predicate, no branch).
  int abase[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    int pix = 16 * m + lp;
    pix = pix < npix_out ? pix : npix_out - 1;
    const int oy = pix / g.Wo, ox = pix - oy * g.Wo;
    abase[m] = (oy * STRIDE) * row_stride + (ox * STRIDE) * P4 + lg;
  }

  // Frames b, b + gridDim.x, ...: while frame i is computed out of LDS, frame i+1 is on its way
  // into registers; two barriers per frame hand the LDS image over.
  u32x4 v[NV];
  int b = blockIdx.x;
  {
    const u32x4* src = g.in + (size_t)b * total;
#pragma unroll
    for (int u = 0; u < NV; ++u) v[u] = src[piece(u)];
  }
  for (; b < g.B; b += gridDim.x) {
#pragma unroll
    for (int u = 0; u < NV; ++u) img[lds_idx[u]] = v[u];
    __syncthreads();
    {  // the next frame (the last round reads its own frame again; nothing is done with it)
      const int bn = b + (int)gridDim.x < g.B ? b + (int)gridDim.x : b;
      const u32x4* src = g.in + (size_t)bn * total;
#pragma unroll
      for (int u = 0; u < NV; ++u) v[u] = src[piece(u)];
    }

    f32x4 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    // K loop, fully unrolled over the filter taps.  One set of pixel fragments: the fragment of
    // (tap g+1, tile m) is requested right behind the MFMA of (tap g, tile m), which has read
    // its operands by the time the data comes back, i.e. MT MFMAs ahead of its use.
    u32x4 pf[MT];
    auto tap_off = [&](int gi) { return (gi / KS) * row_stride + (gi % KS) * P4; };
#pragma unroll
    for (int m = 0; m < MT; ++m) pf[m] = img[abase[m] + tap_off(0)];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
      const int off_next = tap_off(gi + 1 < G ? gi + 1 : gi);
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[gi]),
                                                         __builtin_bit_cast(bf16x8, pf[m]), acc[m], 0, 0, 0);
        if (gi + 1 < G) pf[m] = img[abase[m] + off_next];
        __builtin_amdgcn_sched_barrier(0);  // (left alone, the scheduler sinks each read to its use)
      }
    }

    // epilogue: register r of tile m holds channel ntile*16 + 4*lg + r of pixel 16m + lp
    uint16_t* dst = g.out + (size_t)b * npix_out * g.N + ntile * 16 + 4 * lg;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      int pix = 16 * m + lp;
      pix = pix < npix_out ? pix : npix_out - 1;
      float r[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        r[t] = acc[m][t] + bias4[t];
        if (g.relu) r[t] = fmaxf(r[t], 0.0f);
      }
      const f32x2 lo = {r[0], r[1]}, hi = {r[2], r[3]};
      u32x2 o;
      o[0] = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
      o[1] = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
      *(u32x2*)(dst + pix * g.N) = o;
    }
    __syncthreads();  // every wave is done with this frame's image
  }
}

// Row padding in pieces: stride * row pitch = stride * P4 * Wo modulo 16, i.e. (stride 2)
// row pitch = P4 * Wo modulo 8.
int image_row_pad(int W, int Wo) {
  const int P4 = 5;
  return (((P4 * (Wo - W)) % 8) + 8) % 8;
}
size_t image_lds_bytes(int H, int W, int Wo) { return 16 * (size_t)H * (W * 5 + image_row_pad(W, Wo)); }

template <int KS, int STRIDE, int MT>
hipError_t launch_t(const ImageArgs& g, size_t lds, hipStream_t st) {
  // two workgroups per CU (register-resident filter bank), each walking its share of the frames
  const unsigned nb = (unsigned)(g.B < 512 ? g.B : 512);
  conv_image_bf16_kernel<KS, STRIDE, MT><<<dim3(nb, (unsigned)(g.N / 64)), 256, lds, st>>>(g);
  return hipGetLastError();
}

}  // namespace

// Shapes with an instantiation: 4x4 / stride 2 on 32 channels, no padding, output channels a
// multiple of 64, 97..128 output pixels per frame, image within 52 KB of LDS.
bool conv_image_bf16_supported(int Cin, int ksize, int stride, int pad, int H, int W, int Ho, int Wo,
                               int N) {
  if (!(Cin == 32 && ksize == 4 && stride == 2 && pad == 0 && (N % 64) == 0)) return false;
  const int mt = (Ho * Wo + 15) / 16;
  if (mt != 7 && mt != 8) return false;
  return image_lds_bytes(H, W, Wo) <= kMaxLds && H * W * 4 <= 9 * 256;
}

// Lane fragments of the weights (bf16 bits, rounded to nearest even):
// wpk[(((ntile*G + tap)*64 + lane)*8 + e] = W[ntile*16 + lane%16][c = 8*(lane/16) + e][p][q],
// tap = p*ksize + q.  w: [cout][cin = 32][k][k].
void conv_image_bf16_pack(const float* w, int cout, int k, std::vector<uint16_t>& wpk) {
  const int cin = 32, G = k * k;
  wpk.assign((size_t)cout * cin * k * k, 0);
  for (int nt = 0; nt < cout / 16; ++nt)
    for (int tap = 0; tap < G; ++tap)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int p = tap / k, q = tap % k;
          const int c = 8 * (lane / 16) + e;
          const int n = nt * 16 + lane % 16;
          const float f = w[(((size_t)n * cin + c) * k + p) * k + q];
          uint32_t u;
          memcpy(&u, &f, 4);
          wpk[(((size_t)nt * G + tap) * 64 + lane) * 8 + e] =
              (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
        }
}

// in: bf16 [B][H][W][32]; out: bf16 [B][Ho*Wo][N]; bias fp32 [N].
hipError_t launch_conv_image_bf16(const void* in, const uint16_t* wpk, const float* bias, void* out,
                                  int B, int H, int W, int Cin, int ksize, int stride, int Ho,
                                  int Wo, int N, int relu, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (!conv_image_bf16_supported(Cin, ksize, stride, 0, H, W, Ho, Wo, N)) return hipErrorInvalidValue;
  if ((H - ksize) / stride + 1 != Ho || (W - ksize) / stride + 1 != Wo) return hipErrorInvalidValue;
  ImageArgs g;
  g.in = (const u32x4*)in; g.wpk = (const u32x4*)wpk; g.bias = bias; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.Ho = Ho; g.Wo = Wo; g.N = N; g.relu = relu;
  g.row_pad = image_row_pad(W, Wo);
  const size_t lds = image_lds_bytes(H, W, Wo);
  const int mt = (Ho * Wo + 15) / 16;
  if (H * W * 4 > 9 * 256) return hipErrorInvalidValue;  // pieces per thread
  return mt == 7 ? launch_t<4, 2, 7>(g, lds, st) : launch_t<4, 2, 8>(g, lds, st);
}

}  // namespace sf

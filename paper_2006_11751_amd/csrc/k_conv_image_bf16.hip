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
// The third convolution (3x3 / stride 2 on 64 channels, 18 output pixels per frame) takes four
// frames per round (72 pixels = 4.5 tiles) in workgroups of eight waves, one 16-channel tile
// each (18 K groups: 72 registers of filter bank per lane).
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
  const u32x4* in;    // bf16 [B][H][W][CIN], CIN/8 pieces per pixel
  const u32x4* wpk;   // [N/16][G][64] lane fragments, G = KS*KS*CIN/32
  const float* bias;  // [N]
  uint16_t* out;      // bf16 [B][Ho*Wo][N]
  int B, H, W, Ho, Wo, N, relu;
  int row_pad;        // 16-byte pieces appended to every image row in LDS
  int frame_pad;      // ... and to every frame
};

// CIN input channels (32 or 64: one or two K groups per filter tap), FR frames per round of a
// workgroup (their output pixels, FR*Ho*Wo <= 16*MT, form one row-major sequence that is cut
// into MT 16-pixel tiles), NPW 16-channel tiles per wave (a workgroup covers 64*NPW output
// channels), WRES: the wave's filter bank stays in registers (else its fragments stream from
// memory two groups ahead), NV: image pieces per thread and round, NW: waves per workgroup.
template <int CIN, int KS, int STRIDE, int FR, int MT, int NPW, bool WRES, int NV, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void conv_image_bf16_kernel(ImageArgs g) {
  constexpr int NT = 64 * NW;      // threads
  constexpr int C4 = CIN / 8;      // 16-byte pieces per pixel
  constexpr int P4 = C4 + 1;       // LDS pixel pitch in pieces (odd)
  constexpr int HALVES = CIN / 32; // K groups per filter tap
  constexpr int G = KS * KS * HALVES;
  extern __shared__ __attribute__((aligned(16))) u32x4 img[];  // [FR][frame_stride] pieces

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lp = lane & 15, lg = lane >> 4;
  const int nt0 = ((int)blockIdx.y * NW + wave) * NPW;  // first 16-channel tile of the wave
  const int npix_out = g.Ho * g.Wo;
  const int frame_pieces = g.H * g.W * C4;
  const int row_stride = g.W * P4 + g.row_pad;
  const int frame_stride = g.H * row_stride + g.frame_pad;
  const int full_pieces = FR * frame_pieces, full_pix = FR * npix_out;

  // The wave's fragments start at a wave-uniform address (kept in scalar registers, so that
  // the unrolled K loop does not hold one vector address pair per fragment); fragment (j, gi)
  // of this lane is at byte (j*G + gi)*1024 + lane*16.
  typedef const __attribute__((address_space(1))) unsigned char* global_bytes;
  typedef const __attribute__((address_space(1))) u32x4* global_u32x4;
  global_bytes wbase;
  {
    const uintptr_t a = (uintptr_t)(g.wpk + (size_t)nt0 * G * 64);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    wbase = (global_bytes)(((uintptr_t)hi << 32) | lo);
  }
  const unsigned lane_off = (unsigned)lane * 16u;
  auto wfrag = [&](int j, int gi) -> u32x4 {
    return *(global_u32x4)(wbase + (size_t)((j * G + gi) * 1024) + lane_off);
  };
  u32x4 wf[WRES ? G : 3][NPW];
  if (WRES) {
#pragma unroll
    for (int t = 0; t < G; ++t)
#pragma unroll
      for (int j = 0; j < NPW; ++j) wf[t][j] = wfrag(j, t);
  }
  f32x4 bias4[NPW];
#pragma unroll
  for (int j = 0; j < NPW; ++j) bias4[j] = *(const f32x4*)(g.bias + (nt0 + j) * 16 + 4 * lg);

  // this thread's pieces of a round's images: LDS index (past the end: the last piece again)
  int lds_idx[NV];
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    int f = tid + NT * u;
    f = f < full_pieces ? f : full_pieces - 1;
    const int fr = f / frame_pieces, r = f - fr * frame_pieces;
    const int pix = r / C4, c4 = r - pix * C4;
    const int y = pix / g.W, x = pix - y * g.W;
    lds_idx[u] = fr * frame_stride + y * row_stride + x * P4 + c4;
  }
  // this lane's pixel of every tile: LDS index of its window's first pixel plus the lane
  // group's channel piece.  Pixels past the end repeat the last one (computed again, stored
  // again with the same bits: no per-lane predicate, no branch).
  int abase[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    int n = 16 * m + lp;
    n = n < full_pix ? n : full_pix - 1;
    const int fr = n / npix_out, pix = n - fr * npix_out;
    const int oy = pix / g.Wo, ox = pix - oy * g.Wo;
    abase[m] = fr * frame_stride + (oy * STRIDE) * row_stride + (ox * STRIDE) * P4 + lg;
  }

  // Rounds it, it + gridDim.x, ...: while round i is computed out of LDS, the images of the
  // workgroup's next round are on their way into registers; two barriers per round hand the
  // LDS over.  A last round with fewer than FR frames re-reads its last valid piece instead of
  // reading past the batch, and stores under a predicate.
  const int n_rounds = (g.B + FR - 1) / FR;
  u32x4 v[NV];
  auto load_round = [&](int it) {
    const int frames = g.B - it * FR < FR ? g.B - it * FR : FR;
    const int valid = frames * frame_pieces;
    const u32x4* src = g.in + (size_t)it * full_pieces;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int f = tid + NT * u;
      v[u] = src[f < valid ? f : valid - 1];
    }
  };
  int it = blockIdx.x;
  load_round(it);
  for (; it < n_rounds; it += gridDim.x) {
#pragma unroll
    for (int u = 0; u < NV; ++u) img[lds_idx[u]] = v[u];
    __syncthreads();
    load_round(it + (int)gridDim.x < n_rounds ? it + (int)gridDim.x : it);  // (last: its own again)
    if (!WRES) {
#pragma unroll
      for (int j = 0; j < NPW; ++j) {
        wf[0][j] = wfrag(j, 0);
        wf[1][j] = wfrag(j, 1);
      }
    }

    f32x4 acc[MT][NPW];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int j = 0; j < NPW; ++j) acc[m][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    // K loop, fully unrolled over the K groups.  One set of pixel fragments: the fragment of
    // (group g+1, tile m) is requested right behind the MFMAs of (group g, tile m), which have
    // read their operands by the time the data comes back, i.e. MT tiles ahead of its use.
    u32x4 pf[MT];
    if constexpr (WRES) {
      auto grp_off = [&](int gi) {
        const int tap = gi / HALVES, half = gi - tap * HALVES;
        return (tap / KS) * row_stride + (tap % KS) * P4 + 4 * half;
      };
#pragma unroll
      for (int m = 0; m < MT; ++m) pf[m] = img[abase[m] + grp_off(0)];
#pragma unroll
      for (int gi = 0; gi < G; ++gi) {
        const int off_next = grp_off(gi + 1 < G ? gi + 1 : gi);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
          for (int j = 0; j < NPW; ++j)
            acc[m][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, wf[gi][j]), __builtin_bit_cast(bf16x8, pf[m]), acc[m][j], 0, 0, 0);
          if (gi + 1 < G) pf[m] = img[abase[m] + off_next];
          __builtin_amdgcn_sched_barrier(0);  // (left alone, the scheduler sinks each read to its use)
        }
      }
    } else {
      // Streamed weights: the loop over filter rows stays a loop (unrolled, every fragment
      // would keep a vector address pair alive across the rounds); a row's KS*HALVES groups are
      // unrolled, their count a multiple of the three-deep fragment ring.  The fragment two
      // groups ahead is requested at the start of a group (past the end: the last one again).
      constexpr int RG = KS * HALVES;  // groups per filter row
      static_assert(WRES || RG % 3 == 0, "fragment ring of three");
#pragma unroll
      for (int m = 0; m < MT; ++m) pf[m] = img[abase[m]];
      int row_off = 0;
#pragma unroll 1
      for (int p = 0; p < KS; ++p) {
        const int next_row = p + 1 < KS ? row_off + row_stride : row_off;
#pragma unroll
        for (int sg = 0; sg < RG; ++sg) {
          {
            int gn = p * RG + sg + 2;
            gn = gn < G ? gn : G - 1;
#pragma unroll
            for (int j = 0; j < NPW; ++j) wf[(sg + 2) % 3][j] = wfrag(j, gn);
          }
          // LDS offset of the next group: the next piece pair of this row, or the next row
          const int qn = (sg + 1) / HALVES, hn = (sg + 1) % HALVES;
          const int off_next = sg + 1 < RG ? row_off + qn * P4 + 4 * hn : next_row;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int j = 0; j < NPW; ++j)
              acc[m][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  __builtin_bit_cast(bf16x8, wf[sg % 3][j]), __builtin_bit_cast(bf16x8, pf[m]), acc[m][j], 0, 0, 0);
            pf[m] = img[abase[m] + off_next];  // (after the last group: read again, unused)
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        row_off = next_row;
      }
    }

    // epilogue: register r of (tile m, channel tile j) holds channel (nt0+j)*16 + 4*lg + r of
    // output pixel 16m + lp of the round
    const int frames = g.B - it * FR < FR ? g.B - it * FR : FR;
    const int nvalid = frames * npix_out;
    uint16_t* dst = g.out + (size_t)it * full_pix * g.N + nt0 * 16 + 4 * lg;
    auto write_out = [&](auto checked) {
      constexpr bool CHECK = decltype(checked)::value;
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        int n = 16 * m + lp;
        const bool live = n < nvalid;
        n = n < full_pix ? n : full_pix - 1;
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
          float r[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            r[t] = acc[m][j][t] + bias4[j][t];
            if (g.relu) r[t] = fmaxf(r[t], 0.0f);
          }
          const f32x2 lo = {r[0], r[1]}, hi = {r[2], r[3]};
          u32x2 o;
          o[0] = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
          o[1] = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
          if (!CHECK || live) *(u32x2*)(dst + (size_t)n * g.N + j * 16) = o;
        }
      }
    };
    if (frames == FR)
      write_out(std::false_type{});
    else
      write_out(std::true_type{});
    __syncthreads();  // every wave is done with this round's images
  }
}

// Padding in pieces.  With neighbouring output pixels STRIDE * P4 = 2 * P4 pieces apart, output
// pixel n of a round reads piece 2 * P4 * n + const modulo 16 throughout if
//   row pitch   = P4 * Wo         modulo 8,
//   frame pitch = 2 * P4 * Ho*Wo  modulo 16.
struct ImageLayout {
  int row_pad, frame_pad;
  size_t lds_bytes;
};
ImageLayout image_layout(int Cin, int FR, int H, int W, int Ho, int Wo) {
  const int P4 = Cin / 8 + 1;
  ImageLayout L;
  L.row_pad = (((P4 * Wo - W * P4) % 8) + 8) % 8;
  const int row = W * P4 + L.row_pad;
  L.frame_pad = FR > 1 ? (((2 * P4 * Ho * Wo - H * row) % 16) + 16) % 16 : 0;
  L.lds_bytes = 16 * (size_t)FR * (H * row + L.frame_pad);
  return L;
}

// which instantiation takes a layer: 0 none; 1, 2: 4x4 / stride 2 on 32 channels, one frame per
// round in 7 or 8 pixel tiles; 3: 3x3 / stride 2 on 64 channels, four frames per round in 5 tiles
int image_variant(int Cin, int ksize, int stride, int pad, int H, int W, int Ho, int Wo, int N) {
  if (stride != 2 || pad != 0) return 0;
  if (Cin == 32 && ksize == 4 && (N % 64) == 0) {
    const int mt = (Ho * Wo + 15) / 16;
    if ((mt == 7 || mt == 8) && H * W * 4 <= 9 * 256 &&
        image_layout(Cin, 1, H, W, Ho, Wo).lds_bytes <= kMaxLds)
      return mt == 7 ? 1 : 2;
  }
  if (Cin == 64 && ksize == 3 && (N % 128) == 0) {
    if (4 * Ho * Wo > 64 && 4 * Ho * Wo <= 80 && 4 * H * W * 8 <= 7 * 512 &&
        image_layout(Cin, 4, H, W, Ho, Wo).lds_bytes <= kMaxLds)
      return 3;
  }
  return 0;
}

template <int CIN, int KS, int FR, int MT, int NPW, bool WRES, int NV, int NW>
hipError_t launch_t(ImageArgs g, hipStream_t st) {
  const ImageLayout L = image_layout(CIN, FR, g.H, g.W, g.Ho, g.Wo);
  g.row_pad = L.row_pad;
  g.frame_pad = L.frame_pad;
  // eight waves per CU (two workgroups of four or one of eight), each workgroup walking its
  // share of the rounds
  const int n_rounds = (g.B + FR - 1) / FR;
  const int slots = NW == 4 ? 512 : 256;
  const unsigned nb = (unsigned)(n_rounds < slots ? n_rounds : slots);
  conv_image_bf16_kernel<CIN, KS, 2, FR, MT, NPW, WRES, NV, NW>
      <<<dim3(nb, (unsigned)(g.N / (16 * NW * NPW))), 64 * NW, L.lds_bytes, st>>>(g);
  return hipGetLastError();
}

}  // namespace

bool conv_image_bf16_supported(int Cin, int ksize, int stride, int pad, int H, int W, int Ho, int Wo,
                               int N) {
  return image_variant(Cin, ksize, stride, pad, H, W, Ho, Wo, N) != 0;
}

// Lane fragments of the weights (bf16 bits, rounded to nearest even):
// wpk[(((ntile*G + gi)*64 + lane)*8 + e] = W[ntile*16 + lane%16][c = 32*half + 8*(lane/16) + e]
// [p][q], gi = (p*ksize + q) * (cin/32) + half.  w: [cout][cin][k][k].
void conv_image_bf16_pack(const float* w, int cout, int cin, int k, std::vector<uint16_t>& wpk) {
  const int halves = cin / 32, G = k * k * halves;
  wpk.assign((size_t)cout * cin * k * k, 0);
  for (int nt = 0; nt < cout / 16; ++nt)
    for (int gi = 0; gi < G; ++gi)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int tap = gi / halves, half = gi % halves;
          const int p = tap / k, q = tap % k;
          const int c = 32 * half + 8 * (lane / 16) + e;
          const int n = nt * 16 + lane % 16;
          const float f = w[(((size_t)n * cin + c) * k + p) * k + q];
          uint32_t u;
          memcpy(&u, &f, 4);
          wpk[(((size_t)nt * G + gi) * 64 + lane) * 8 + e] =
              (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
        }
}

// in: bf16 [B][H][W][Cin]; out: bf16 [B][Ho*Wo][N]; bias fp32 [N].
hipError_t launch_conv_image_bf16(const void* in, const uint16_t* wpk, const float* bias, void* out,
                                  int B, int H, int W, int Cin, int ksize, int stride, int Ho,
                                  int Wo, int N, int relu, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if ((H - ksize) / stride + 1 != Ho || (W - ksize) / stride + 1 != Wo) return hipErrorInvalidValue;
  ImageArgs g;
  g.in = (const u32x4*)in; g.wpk = (const u32x4*)wpk; g.bias = bias; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.Ho = Ho; g.Wo = Wo; g.N = N; g.relu = relu;
  g.row_pad = g.frame_pad = 0;
  switch (image_variant(Cin, ksize, stride, 0, H, W, Ho, Wo, N)) {
    case 1: return launch_t<32, 4, 1, 7, 1, true, 9, 4>(g, st);
    case 2: return launch_t<32, 4, 1, 8, 1, true, 9, 4>(g, st);
    case 3: return launch_t<64, 3, 4, 5, 1, true, 7, 8>(g, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sf

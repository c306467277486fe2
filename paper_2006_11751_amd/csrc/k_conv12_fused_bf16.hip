// First and second convolution of the plain encoder in bf16 configurations as one kernel
// (paper, App. "Model architectures": the convolutional encoder), so that the first layer's
// output (the largest tensor of the step: 17 x 31 x 32 values per frame) never leaves the
// compute unit.  Run as two launches, the first layer writes 138 MB at B = 4096 and the second
// reads them straight back: 45 % of the step's HBM traffic.
//
// A workgroup of four waves walks frames b, b + gridDim.x, ...  Per frame:
//   1. the planar byte frame (3 x 72 x 128 = 27 KB), fetched into registers during the previous
//      frame, goes to LDS; barrier;
//   2. the next frame's bytes are requested;
//   3. first convolution, 8x8 / stride 4 -> 32 channels, on the int8 MFMA against the
//      fixed-point digit planes of its filter bank (two planes; see k_conv1_i8.hip for the
//      arithmetic): wave w computes output rows w, w + 4, ...; its ReLU'd bf16 results go into a
//      channels-last image in LDS (pixel pitch 64 + 16 bytes, rows padded: the layout of
//      k_conv_image_bf16.hip); barrier;
//   4. second convolution, 4x4 / stride 2 -> 64 channels, on v_mfma_f32_16x16x32_bf16 out of
//      that image: wave w owns output channels 16w .. 16w + 15 and all MT 16-pixel tiles of the
//      frame, its filter bank (16 taps x 16 bytes per lane) staying in registers; bias, ReLU,
//      bf16, one 8-byte store of four channels per lane and tile.
// The MFMA sequences, epilogues and roundings are those of the two separate kernels, so the
// results are the same bits.  LDS: 27 KB + 42 KB per workgroup, two workgroups per CU.
//
// v_mfma_i32_32x32x32_i8: lane l supplies 16 bytes A[i = l%32][k = 16*(l/32) + e] and
// B[k][j = l%32]; D[i][j]: j = l%32, i = (v%4) + 8*(v/4) + 4*(l/32) in register v.
// v_mfma_f32_16x16x32_bf16: lane l supplies A[i = l%16][k = 8*(l/16) + e] and
// B[k][j = l%16] (16 bytes each); D[i][j] sits in lane j + 16*(i/4), register i%4.
#include <mutex>
#include <type_traits>

#include "sf_internal.h"

namespace sf {

namespace {

typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kNT = 64 * kWaves;
constexpr int kK1 = 8, kS1 = 4, kC1 = 32;  // first layer: filter, stride, output channels
constexpr int kK2 = 4, kS2 = 2;            // second layer: filter, stride (64 output channels)
constexpr int kP4 = kC1 / 8 + 1;           // LDS pixel pitch of the bf16 image in 16-byte pieces
constexpr int kNV = 7;                     // 16-byte pieces of a byte frame per thread
constexpr float kInvRadix = 1.0f / 254.0f;

struct __attribute__((packed, aligned(4))) U2 {
  uint32_t x, y;
};

struct Conv12Args {
  const uint8_t* obs;   // [B][3][H][W] bytes
  const int* wpk1;      // digit planes of the first filter bank, lane order
  const float* scale1;  // [32]
  const float* bias1;   // [32]
  const u32x4* wpk2;    // [4][16][64] lane fragments of the second filter bank
  const float* bias2;   // [64]
  uint16_t* out;        // bf16 [B][Ho2*Wo2][64]
  int B, H, W, Ho1, Wo1, Ho2, Wo2;
  int row_stride;       // image row pitch in pieces
  int frame_lds_bytes;  // byte frame rounded up to 16
};

template <int MT>
__global__ __launch_bounds__(kNT, 2) void conv12_fused_bf16_kernel(Conv12Args g) {
  constexpr int CIN = 3;
  constexpr int NSTEP = CIN * kK1 / 4;  // int8 MFMA K steps of the first layer
  constexpr int G = kK2 * kK2;          // filter taps of the second layer (one K group each)
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  uint8_t* frame_lds = lds;
  u32x4* img = (u32x4*)(lds + g.frame_lds_bytes);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int n = lane & 31, h = lane >> 5;   // first layer: channel / lane half
  const int lp = lane & 15, lg = lane >> 4; // second layer: pixel of a tile / channel piece

  // ---- operands that stay in registers while the workgroup walks its frames ----
  i32x4 wd[NSTEP][2];
#pragma unroll
  for (int s = 0; s < NSTEP; ++s)
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
      for (int w = 0; w < 4; ++w) wd[s][d][w] = g.wpk1[((s * 3 + d) * 4 + w) * 64 + lane];
  const float s_n = g.scale1[n], b_n = g.bias1[n];
  u32x4 wf[G];
#pragma unroll
  for (int t = 0; t < G; ++t) wf[t] = g.wpk2[((size_t)wv * G + t) * 64 + lane];
  const f32x4 bias4 = *(const f32x4*)(g.bias2 + wv * 16 + 4 * lg);

  const int frame_bytes = CIN * g.H * g.W;
  const int pieces = frame_bytes / 16;
  const int row_stride = g.row_stride;

  // first layer: LDS byte offsets of this lane's two 8-byte runs per MFMA step at output row 0
  // ((channel, filter row) group 4s + 2h + pp, output pixel n; lanes past the row end repeat
  // the last pixel), and of its eight image words (tile row (v%4) + 8(v/4) + 4h, channel pair
  // n & ~1; the even lane keeps tile rows v = 2k, the odd lane v = 2k + 1)
  // (group 4s + 2h + pp = channel s/2, filter row 4(s%2) + 2h + pp: a per-lane base plus
  // offsets that are the same for all lanes)
  const int ox1 = n < g.Wo1 ? n : g.Wo1 - 1;
  const uint32_t gbase = (uint32_t)(2 * h * g.W + ox1 * kS1);
  // word k of the lane: tile row v = 2k + (n & 1), i.e. pixel (n & 1) + 4h + 2(k & 1) + 8(k >> 1):
  // a per-lane base plus a constant.  Image rows hold 32 pixels, so tile rows past the end of the
  // output row (copies of its last pixel) land in pixels that nobody reads.
  const uint32_t ibase = (uint32_t)(((n & 1) + 4 * h) * (kP4 * 16) + (n & ~1) * 2);
  // second layer: LDS piece index of this lane's window origin in every pixel tile (pixels
  // past the end repeat the last one: computed and stored again with the same bits)
  const int npix2 = g.Ho2 * g.Wo2;
  int abase[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    int p = 16 * m + lp;
    p = p < npix2 ? p : npix2 - 1;
    const int oy = p / g.Wo2, ox = p - oy * g.Wo2;
    abase[m] = (oy * kS2) * row_stride + (ox * kS2) * kP4 + lg;
  }

  u32x4 fv[kNV];
  auto load_frame = [&](int b) {
    const u32x4* src = (const u32x4*)(g.obs + (size_t)b * frame_bytes);
#pragma unroll
    for (int u = 0; u < kNV; ++u) {
      const int f = tid + kNT * u;
      fv[u] = src[f < pieces ? f : pieces - 1];
    }
  };

  int b = blockIdx.x;
  load_frame(b);
  for (; b < g.B; b += gridDim.x) {
#pragma unroll
    for (int u = 0; u < kNV; ++u) {
      const int f = tid + kNT * u;
      *(u32x4*)(frame_lds + 16 * (size_t)(f < pieces ? f : pieces - 1)) = fv[u];
    }
    __syncthreads();  // frame bytes visible; every wave is past the previous frame's image reads

    // ---- first convolution: rows wv, wv + 4, ... into the LDS image ----
    {
      U2 rb[NSTEP][2];
      auto load_row = [&](int oy) {
        const uint8_t* base = frame_lds + (size_t)(oy * kS1) * g.W;
#pragma unroll
        for (int s = 0; s < NSTEP; ++s)
#pragma unroll
          for (int pp = 0; pp < 2; ++pp)
            rb[s][pp] = *(const U2*)(base + gbase + (uint32_t)(((s / 2) * g.H + 4 * (s % 2) + pp) * g.W));
      };
      int oy = wv;
      if (oy < g.Ho1) load_row(oy);
      for (; oy < g.Ho1; oy += kWaves) {
        i32x16 s1, s2;
#pragma unroll
        for (int v = 0; v < 16; ++v) s1[v] = s2[v] = 0;
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
          i32x4 a;  // byte - 128 on all 16 pixels of the two runs
          a[0] = (int)(rb[s][0].x ^ 0x80808080u);
          a[1] = (int)(rb[s][0].y ^ 0x80808080u);
          a[2] = (int)(rb[s][1].x ^ 0x80808080u);
          a[3] = (int)(rb[s][1].y ^ 0x80808080u);
          s1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][0], s1, 0, 0, 0);
          s2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, wd[s][1], s2, 0, 0, 0);
        }
        // the wave's next row is read behind this row's MFMAs, under its epilogue
        load_row(oy + kWaves < g.Ho1 ? oy + kWaves : oy);
        float r[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float q = fmaf((float)s2[v], kInvRadix, (float)s1[v]);
          r[v] = fmaxf(fmaf(q, s_n, b_n), 0.0f);
        }
        // neighbouring lanes (channels n, n ^ 1) swap half of their rows, so that each writes
        // (channel n & ~1, channel n | 1) pairs as 32-bit words
        uint8_t* row = (uint8_t*)img + (size_t)oy * row_stride * 16;
        const bool odd = (n & 1) != 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float mine = odd ? r[2 * k + 1] : r[2 * k];
          const float give = odd ? r[2 * k] : r[2 * k + 1];
          const float got = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(give), 0xB1, 0xF, 0xF, true));
          const f32x2 pair = {odd ? got : mine, odd ? mine : got};
          *(uint32_t*)(row + ibase + (2 * (k & 1) + 8 * (k >> 1)) * (kP4 * 16)) =
              __builtin_bit_cast(unsigned, __builtin_convertvector(pair, bf16x2));
        }
      }
    }
    __syncthreads();  // the frame's first-layer image is complete
    // the next frame's bytes travel into registers during the second convolution (requested
    // here, not earlier: the first convolution has no registers to spare for them)
    load_frame(b + (int)gridDim.x < g.B ? b + (int)gridDim.x : b);  // (last round: its own again)

    // ---- second convolution out of the image, pixel tiles in two passes (the filter bank is
    // used twice, the accumulators and pixel fragments of a pass are half as many) ----
    // (a frame base that is the same for all lanes plus a 32-bit lane offset: no 64-bit
    // address per tile to keep in registers)
    uint8_t* dst = (uint8_t*)g.out + (size_t)b * npix2 * 128;
    const uint32_t lane_off = (uint32_t)((wv * 16 + 4 * lg) * 2);
    auto tap_off = [&](int t) { return (t / kK2) * row_stride + (t % kK2) * kP4; };
    auto conv2_tiles = [&](auto m0c, auto mnc) {
      constexpr int M0 = decltype(m0c)::value, MN = decltype(mnc)::value;
      f32x4 acc[MN];
      u32x4 pf[MN];
#pragma unroll
      for (int m = 0; m < MN; ++m) {
        acc[m] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        pf[m] = img[abase[M0 + m]];
      }
#pragma unroll
      for (int t = 0; t < G; ++t) {
        const int off_next = tap_off(t + 1 < G ? t + 1 : t);
#pragma unroll
        for (int m = 0; m < MN; ++m) {
          acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[t]),
                                                           __builtin_bit_cast(bf16x8, pf[m]), acc[m], 0, 0, 0);
          if (t + 1 < G) pf[m] = img[abase[M0 + m] + off_next];
          __builtin_amdgcn_sched_barrier(0);  // (left alone, the scheduler sinks each read to its use)
        }
      }
#pragma unroll
      for (int m = 0; m < MN; ++m) {
        int p = 16 * (M0 + m) + lp;
        p = p < npix2 ? p : npix2 - 1;
        float r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = fmaxf(acc[m][t] + bias4[t], 0.0f);
        const f32x2 lo = {r[0], r[1]}, hi = {r[2], r[3]};
        u32x2 o;
        o[0] = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2));
        o[1] = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2));
        *(u32x2*)(dst + ((uint32_t)p * 128u + lane_off)) = o;
      }
    };
    conv2_tiles(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
    conv2_tiles(std::integral_constant<int, 4>{}, std::integral_constant<int, MT - 4>{});
    // no barrier here: the next frame's bytes go to their own LDS region, and its barrier
    // (which every wave reaches only after these image reads) precedes the next image writes
  }
}

// Image row pitch in pieces: room for 32 pixels, and congruent to kP4 * Wo2 modulo 8 (then
// output pixel n of the second layer reads piece 2 * kP4 * n + const modulo 16 also across the
// end of an output row: no bank conflicts between the 16 pixels of a tile).
int image_row_stride(int Wo2) {
  const int want = (kP4 * Wo2) % 8;
  int r = 32 * kP4;
  while (r % 8 != want) ++r;
  return r;
}

}  // namespace

// Shapes: three byte planes, first layer 8x8 / 4 -> 32 channels in one 32-pixel chunk per
// output row, second layer 4x4 / 2 -> 64 channels with seven 16-pixel tiles, both without padding
// and with ReLU; frame a multiple of 16 bytes, at most 28 KB; LDS for two workgroups per CU.
bool conv12_fused_bf16_supported(int cin, int H, int W, const sf_conv& c1, const sf_conv& c2) {
  if (cin != 3 || c1.k != kK1 || c1.stride != kS1 || c1.pad != 0 || c1.cout != kC1) return false;
  if (c2.k != kK2 || c2.stride != kS2 || c2.pad != 0 || c2.cout != 64) return false;
  if (W % 4 != 0 || H < kK1 || W < kK1) return false;
  const int Ho1 = (H - kK1) / kS1 + 1, Wo1 = (W - kK1) / kS1 + 1;
  if (Wo1 > 32 || Ho1 < kK2 || Wo1 < kK2) return false;
  const int Ho2 = (Ho1 - kK2) / kS2 + 1, Wo2 = (Wo1 - kK2) / kS2 + 1;
  // seven 16-pixel tiles (a byte frame of at most 28 KB has no room for more)
  if ((Ho2 * Wo2 + 15) / 16 != 7) return false;
  const int frame_bytes = cin * H * W;
  if (frame_bytes % 16 != 0 || frame_bytes > kNV * kNT * 16) return false;
  const size_t lds = (size_t)frame_bytes + 16 * (size_t)Ho1 * image_row_stride(Wo2);
  return lds <= 80 * 1024;
}

// L1, L2: the two layers as executed separately (L1's digit planes, scales and bias, L2's
// image-kernel fragments and bias); out: bf16 [B][Ho2*Wo2][64].
hipError_t launch_conv12_fused_bf16(const ConvLayer& L1, const ConvLayer& L2, int B, const uint8_t* obs,
                                    void* out, hipStream_t st) {
  if (B == 0) return hipSuccess;
  if (((uintptr_t)obs & 15) != 0 || L1.planes != 2) return hipErrorInvalidValue;
  Conv12Args g;
  g.obs = obs; g.wpk1 = L1.ipk; g.scale1 = L1.spk; g.bias1 = L1.bpk8;
  g.wpk2 = (const u32x4*)L2.wbf; g.bias2 = L2.bbf; g.out = (uint16_t*)out;
  g.B = B; g.H = L1.H; g.W = L1.W; g.Ho1 = L1.Ho; g.Wo1 = L1.Wo; g.Ho2 = L2.Ho; g.Wo2 = L2.Wo;
  g.row_stride = image_row_stride(L2.Wo);
  g.frame_lds_bytes = L1.cin * L1.H * L1.W;
  const size_t lds = (size_t)g.frame_lds_bytes + 16 * (size_t)L1.Ho * g.row_stride;
  if ((L2.Ho * L2.Wo + 15) / 16 != 7) return hipErrorInvalidValue;
  auto kern = conv12_fused_bf16_kernel<7>;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&] {
    attr_status = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
  });
  if (attr_status != hipSuccess) return attr_status;
  // two workgroups per CU, each walking its share of the frames
  const int blocks = B < 512 ? B : 512;
  kern<<<blocks, kNT, lds, st>>>(g);
  return hipGetLastError();
}

}  // namespace sf

// First convolution of the residual encoder (3x3, stride 1, pad 1, bytes in, normalised on the
// way in) and the 3x3 / stride 2 / pad 1 max-pool behind it, 16 output channels, fp16 out (the
// encoder follows IMPALA; paper, App. DMLab-30).
//
// The full-resolution convolution output is never stored, not even in LDS: rounding to fp16 is
// monotone, so the maximum of the rounded values is the rounded maximum, and the pool runs on
// the fp32 accumulators.  The lanes of a 16-pixel MFMA tile stand for 16 neighbouring POOLED
// columns x, and the three convolution columns 2x-1, 2x, 2x+1 of a pooled pixel are three
// tiles of the same lane, so the horizontal maximum is lane-local.  A wave walks down the
// pooled rows of its column group and carries convolution row 2y+1 (which rows y and y+1
// share) in registers, so the vertical maximum is lane-local too.  Per pooled row a wave
// computes two convolution rows of three tiles: convolution columns 2x-1 and 2x+1 are both
// computed (1.5 x the MFMA work) instead of being shifted across lanes.
//
// The frame sits in LDS as fp16 pixels of four channels (three and a zero), 8 bytes each, with
// a zero ring (two columns left and right, one row above and below).  K = 32 of an MFMA is two
// filter rows x four window columns x four channels; a 3-wide filter occupies columns 0..2 of
// the window ("lo" bank) or columns 1..3 ("hi" bank), the fourth having zero weights.  With
// the window of pooled column x starting at image column 2x-2 (16-byte aligned), convolution
// column 2x-1 is the lo bank and column 2x the hi bank on the SAME pixel operand, and column
// 2x+1 is the lo bank on the window 16 bytes further on.  A second MFMA covers the third filter
// row (its upper K half has zero weights and re-reads the same pixels).
//
// v_mfma_f32_16x16x32_f16: lane l supplies A[i = l%16][k = 8*(l/16) + e] and
// B[k = 8*(l/16) + e][j = l%16]; D[i][j] sits in lane j + 16*(i/4), register i%4.
// A = weights (i = output channel), B = pixels (j = pooled column).
//
// A workgroup of eight waves walks frames; the next frame's bytes are in flight while the
// current one is computed.  Two workgroups share a CU, so one's staging overlaps the other's
// MFMAs.
#include <mutex>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kNW = 8, kNT = 64 * kNW;
constexpr int kMaxIt = 5;                 // four-pixel items per thread and frame
constexpr size_t kMaxLds = 80 * 1024;     // two workgroups per CU

__device__ inline unsigned f16_bits(float f) {
  return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);
}
__device__ inline unsigned pack_f16(float a, float b) { return f16_bits(a) | (f16_bits(b) << 16); }
__device__ inline f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b),
                                                c, 0, 0, 0);
}
// Lane-wise maximum of three accumulator quads that MFMAs have just written.  fmaxf would
// canonicalise every operand first (a move each), so this is v_max3_f32 by hand; and because
// the compiler pads the MFMA-to-VALU read hazard only for instructions it has selected itself,
// the wait states travel with the instructions (12: enough for an MFMA of up to eight passes).
__device__ inline f32x4 max3_after_mfma(const f32x4& a, const f32x4& b, const f32x4& c) {
  f32x4 d;
  asm("s_nop 7\n\ts_nop 3\n\t"
      "v_max3_f32 %0, %4, %8, %12\n\t"
      "v_max3_f32 %1, %5, %9, %13\n\t"
      "v_max3_f32 %2, %6, %10, %14\n\t"
      "v_max3_f32 %3, %7, %11, %15"
      : "=&v"(d[0]), "=&v"(d[1]), "=&v"(d[2]), "=&v"(d[3])
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(b[0]), "v"(b[1]), "v"(b[2]), "v"(b[3]), "v"(c[0]),
        "v"(c[1]), "v"(c[2]), "v"(c[3]));
  return d;
}
// The same on values that VALU instructions produced (no hazard).
__device__ inline float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

struct StemPoolArgs {
  const uint8_t* obs;  // planar bytes [B][3][H][W]
  const u32x4* wpk;    // A operands [4][64]: lo rows 0-1, lo row 2, hi rows 0-1, hi row 2
  const float* bias;   // [16] (or longer)
  uint16_t* out;       // fp16 [B][Ho][Wo][16]
  int B, H, W, Ho, Wo;
  int RP;              // LDS row pitch in bytes: (W + 4) pixels of 8 bytes
  int n_cg, n_seg;     // column groups of 16 pooled columns x row segments = a frame's wave units
  int n_items;         // H * W / 4
  float obs_sub, obs_mul;
};

// (second launch bound: waves per SIMD; four = two workgroups of eight waves per CU, 128 VGPRs)
__global__ __launch_bounds__(kNT, 4) void stem_pool_kernel(StemPoolArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char patch[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (scalar: row loops branch uniformly)
  const int j = lane & 15, grp = lane >> 4;
  const size_t plane = (size_t)g.H * g.W;

  // zeros once: the ring is never written again
  for (int i = tid; i < (g.H + 2) * g.RP / 16; i += kNT) ((u32x4*)patch)[i] = u32x4{0u, 0u, 0u, 0u};

  const u32x4 a_lo1 = g.wpk[lane], a_lo2 = g.wpk[64 + lane];
  const u32x4 a_hi1 = g.wpk[128 + lane], a_hi2 = g.wpk[192 + lane];
  const f32x4 bias = *(const f32x4*)(g.bias + 4 * grp);
  // The parameters have arrived before the first frame is requested (vmcnt(0), other counters
  // untouched).  Otherwise the compiler, which must assume their loads pending on some path,
  // drains the load counter ahead of every row loop that uses them, and that wait would catch
  // the next frame's bytes right after they have been requested.
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // Item i = tid + it * kNT is the four pixels at byte 4*i of each colour plane: image row
  // i / (W/4), columns 4*(i % (W/4)) ..; in LDS, row + 1 and column + 2.
  const int Q = g.W >> 2;
  int lds_off[kMaxIt];
#pragma unroll
  for (int it = 0; it < kMaxIt; ++it) {
    const int i = min(tid + it * kNT, g.n_items - 1);
    const int y = i / Q, jq = i - y * Q;
    lds_off[it] = (y + 1) * g.RP + (4 * jq + 2) * 8;
  }
  uint32_t nx[kMaxIt][3];
  auto load_frame = [&](int b) {
    const uint8_t* frame = g.obs + (size_t)b * 3 * plane;
#pragma unroll
    for (int it = 0; it < kMaxIt; ++it) {
      if (it * kNT >= g.n_items) break;  // uniform
      const int i = min(tid + it * kNT, g.n_items - 1);
#pragma unroll
      for (int c = 0; c < 3; ++c) nx[it][c] = *(const uint32_t*)(frame + c * plane + 4 * (size_t)i);
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int it = 0; it < kMaxIt; ++it) {
      if (it * kNT >= g.n_items) break;  // uniform
      float c[4][3];
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int ch = 0; ch < 3; ++ch)
          c[k][ch] = ((float)((nx[it][ch] >> (8 * k)) & 0xFFu) - g.obs_sub) * g.obs_mul;
      const u32x4 lo = {pack_f16(c[0][0], c[0][1]), f16_bits(c[0][2]), pack_f16(c[1][0], c[1][1]),
                        f16_bits(c[1][2])};
      const u32x4 hi = {pack_f16(c[2][0], c[2][1]), f16_bits(c[2][2]), pack_f16(c[3][0], c[3][1]),
                        f16_bits(c[3][2])};
      if (tid + it * kNT < g.n_items) {
        u32x4* dst = (u32x4*)(patch + lds_off[it]);
        dst[0] = lo;
        dst[1] = hi;
      }
    }
  };

  const int n_units = g.n_cg * g.n_seg;
  const float ninf = -__builtin_inff();
  auto compute = [&](int b) {
    for (int u = wave; u < n_units; u += kNW) {
      const int cg = u % g.n_cg, seg = u / g.n_cg;
      const int oy0 = seg * g.Ho / g.n_seg, oy1 = (seg + 1) * g.Ho / g.n_seg;
      const bool live = cg * 16 + j < g.Wo;
      const int x = live ? cg * 16 + j : g.Wo - 1;
      // window of pooled column x: image columns 2x-2 .. 2x+1 = LDS columns 2x .. 2x+3; lane group
      // grp holds columns 2*(grp%2), +1 of filter row grp/2 (first MFMA) or of filter row 2
      const int colb = (2 * x + 2 * (grp & 1)) * 8;
      const unsigned char* p1 = patch + (grp >> 1) * g.RP + colb;
      const unsigned char* p2 = patch + 2 * g.RP + colb;
      // pixel operands of convolution row r (0 <= r < H): windows 2x-2.. and 2x.., filter rows
      // 0-1 (image rows r-1, r = LDS rows r, r+1) and filter row 2
      auto read_row = [&](int r, u32x4 (&bo)[4]) {
        const unsigned char* q1 = p1 + r * g.RP;
        const unsigned char* q2 = p2 + r * g.RP;
        bo[0] = *(const u32x4*)q1;
        bo[1] = *(const u32x4*)q2;
        bo[2] = *(const u32x4*)(q1 + 16);
        bo[3] = *(const u32x4*)(q2 + 16);
      };
      // horizontal maximum of a convolution row over columns 2x-1 .. 2x+1
      auto row_max = [&](const u32x4 (&bo)[4]) {
        f32x4 tlo = mfma(a_lo1, bo[0], bias);  // column 2x-1
        f32x4 thi = mfma(a_hi1, bo[0], bias);  // column 2x
        f32x4 tnx = mfma(a_lo1, bo[2], bias);  // column 2x+1
        tlo = mfma(a_lo2, bo[1], tlo);
        thi = mfma(a_hi2, bo[1], thi);
        tnx = mfma(a_lo2, bo[3], tnx);
        // (column -1 is the pool's padding: the window's own column 0 stands in)
        if (cg == 0) {  // uniform
#pragma unroll
          for (int e = 0; e < 4; ++e) tlo[e] = x == 0 ? thi[e] : tlo[e];
        }
        return max3_after_mfma(tlo, thi, tnx);
      };
      // The operands of a row are requested one row ahead (two register sets: even rows in be,
      // odd rows in bo), so that an LDS read has the previous row's MFMAs to complete behind.
      u32x4 be[4], bo[4];
      f32x4 carry = {ninf, ninf, ninf, ninf};  // row -1 is the pool's padding
      if (oy0 > 0) {
        read_row(2 * oy0 - 1, bo);
        read_row(2 * oy0, be);
        carry = row_max(bo);
      } else {
        read_row(0, be);
      }
      uint16_t* dst = g.out + (((size_t)b * g.Ho + oy0) * g.Wo + x) * 16 + 4 * grp;
      for (int oy = oy0; oy < oy1; ++oy) {
        const bool odd_row = 2 * oy + 1 < g.H;  // (false: the last pooled row of an odd height)
        if (odd_row) read_row(2 * oy + 1, bo);
        const f32x4 h0 = row_max(be);
        if (oy + 1 < oy1) read_row(2 * oy + 2, be);
        f32x4 h1 = {ninf, ninf, ninf, ninf};
        if (odd_row) h1 = row_max(bo);
        f32x4 m;
#pragma unroll
        for (int e = 0; e < 4; ++e) m[e] = max3(carry[e], h0[e], h1[e]);
        carry = h1;
        const u32x2 ov = {pack_f16(m[0], m[1]), pack_f16(m[2], m[3])};
        if (live) *(u32x2*)dst = ov;
        dst += (size_t)g.Wo * 16;
      }
    }
  };

  int b = blockIdx.x;
  load_frame(b);
  __syncthreads();  // zeros in place
  for (; b < g.B; b += gridDim.x) {
    stage();
    __syncthreads();
    if (b + (int)gridDim.x < g.B) load_frame(b + (int)gridDim.x);
    compute(b);
    __syncthreads();  // every read of this frame done before the next one is staged
  }
}

size_t stem_pool_lds_bytes(int H, int W) { return (size_t)(H + 2) * (W + 4) * 8; }

int gcd(int a, int b) { return b == 0 ? a : gcd(b, a % b); }

}  // namespace

// 16 output channels; frame width a multiple of 4; the frame within kMaxIt items per thread and
// within the LDS share of a workgroup.
bool stem_pool_supported(int cin, int cout, int H, int W) {
  return cin == 3 && cout == 16 && W % 4 == 0 && H >= 1 && W >= 4 &&
         (long long)H * W / 4 <= (long long)kMaxIt * kNT && stem_pool_lds_bytes(H, W) <= kMaxLds;
}

// A operands: wpk[((a * 64) + lane) * 8 + e], a = 2*bank + m (bank 0 = lo, 1 = hi; m = 0: filter
// rows 0 and 1, m = 1: filter row 2).  Lane l = output channel l%16, lane group l/16; element e =
// window column 2*((l/16)%2) + e/4, channel e%4.  The filter column is the window column (lo) or
// the window column - 1 (hi); everything else is zero.
void stem_pool_pack(const float* w, bool f16, std::vector<uint16_t>& wpk) {
  wpk.assign((size_t)4 * 64 * 8, 0);
  for (int bank = 0; bank < 2; ++bank)
    for (int m = 0; m < 2; ++m)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int n = lane & 15, grp = lane >> 4;
          const int c = e % 4, wc = 2 * (grp & 1) + e / 4;
          const int q = wc - bank;
          const int p = m == 0 ? (grp >> 1) : ((grp >> 1) == 0 ? 2 : -1);
          if (c < 3 && q >= 0 && q < 3 && p >= 0)
            wpk[(((size_t)(2 * bank + m)) * 64 + lane) * 8 + e] =
                conv_weight_bits(w[(((size_t)n * 3 + c) * 3 + p) * 3 + q], f16);
        }
}

// obs: planar bytes [B][3][H][W]; wpk as stem_pool_pack lays it out; bias: 16 floats;
// out: fp16 [B][(H-1)/2+1][(W-1)/2+1][16].
hipError_t launch_stem_pool(const uint8_t* obs, const uint16_t* wpk, const float* bias, void* out, int B,
                            int H, int W, float obs_sub, float obs_mul, hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  if (!stem_pool_supported(3, 16, H, W)) return hipErrorInvalidValue;
  StemPoolArgs g;
  g.obs = obs; g.wpk = (const u32x4*)wpk; g.bias = bias; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.Ho = (H - 1) / 2 + 1; g.Wo = (W - 1) / 2 + 1;
  g.RP = (W + 4) * 8;
  g.n_cg = (g.Wo + 15) / 16;
  // as many row segments as make the units a multiple of the waves, at least two rows each
  int n_seg = kNW / gcd(g.n_cg, kNW);
  if (n_seg > g.Ho / 2) n_seg = g.Ho / 2;
  g.n_seg = n_seg < 1 ? 1 : n_seg;
  g.n_items = H * (W / 4);
  g.obs_sub = obs_sub; g.obs_mul = obs_mul;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&] {
    attr_status = hipFuncSetAttribute((const void*)stem_pool_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)kMaxLds);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int blocks = B < 512 ? B : 512;  // two workgroups per CU, each walking its share of the frames
  stem_pool_kernel<<<blocks, kNT, stem_pool_lds_bytes(H, W), st>>>(g);
  return hipGetLastError();
}

}  // namespace sf

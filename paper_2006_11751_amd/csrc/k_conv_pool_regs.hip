// Stage convolution of the residual encoder (3x3, stride 1, pad 1, 16 or 32 -> 32 channels, fp16
// in and out) and the 3x3 / stride 2 / pad 1 max-pool behind it, for frames whose pooled width is
// at most 32 (the encoder follows IMPALA; paper, App. DMLab-30).
//
// The full-resolution convolution output is never stored.  Rounding to fp16 is monotone, so the
// pool runs on the fp32 accumulators and only pooled values are rounded.  The 32 pixel lanes of
// an MFMA tile stand for the POOLED columns x of a frame row; a convolution row is two tiles, E
// (convolution columns 2x) and O (columns 2x+1).  A wave walks down the pooled rows of its row
// segment: the maximum over the three convolution rows of a pooled row is lane-local in E and
// in O, and convolution row 2y+1, which pooled rows y and y+1 share, is carried in registers.
// What is left per pooled row is max(E[x], O[x], O[x-1]): one lane shift (ds_bpermute) per
// accumulator register.  No convolution value is computed twice, except the one row that two
// neighbouring row segments share.
//
// The frame sits in LDS with even and odd image columns in separate planes (pixel pitch 48
// bytes for 16 channels, 80 for 32: conflict-free 16-byte reads), each with a zero ring, so
// that the lanes of a fragment read neighbouring pixels of one plane: for filter row p the E
// tile takes odd[x-1], even[x], odd[x] and the O tile even[x], odd[x], even[x+1].
//
// v_mfma_f32_32x32x16_f16: lane l supplies A[i = l%32][k = 8*(l/32) + e] and
// B[k = 8*(l/32) + e][j = l%32]; D[i][j] sits in lane j + 32*((i/4)%2), register
// (i%4) + 4*(i/8).  A = weights (i = output channel), B = pixels (j = pooled column).
//
// A workgroup of eight waves walks frames (two at a time where the pooled width is at most 16:
// lanes 16..31 then stand for the second frame); the next frames' pixels are in flight while
// the current ones are computed.
#include <mutex>

#include "sf_internal.h"

namespace sf {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kNW = 8, kNT = 64 * kNW;
constexpr size_t kMaxLds = 160 * 1024;

__device__ inline unsigned f16_bits(float f) {
  return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);
}
__device__ inline unsigned pack_f16(float a, float b) { return f16_bits(a) | (f16_bits(b) << 16); }
__device__ inline f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b),
                                                c, 0, 0, 0);
}

// a <- max(a, b, c) lane-wise on accumulators that MFMAs have just written.  fmaxf would
// canonicalise every operand first (a move each), so this is v_max3_f32 by hand; and because the
// compiler pads the MFMA-to-VALU read hazard only for instructions it has selected itself, the
// wait states travel with the instructions (12: enough for an MFMA of eight passes).  Four
// statements (one takes at most 30 operands), volatile so that they keep their order behind
// the wait states.
#define SF_MAX3_4(NOPS, a, b, c, o)                                                                 \
  asm volatile(NOPS "v_max3_f32 %0, %0, %4, %8\n\tv_max3_f32 %1, %1, %5, %9\n\t"                      \
                    "v_max3_f32 %2, %2, %6, %10\n\tv_max3_f32 %3, %3, %7, %11"                        \
               : "+v"(a[o]), "+v"(a[o + 1]), "+v"(a[o + 2]), "+v"(a[o + 3])                          \
               : "v"(b[o]), "v"(b[o + 1]), "v"(b[o + 2]), "v"(b[o + 3]), "v"(c[o]), "v"(c[o + 1]), \
                 "v"(c[o + 2]), "v"(c[o + 3]))
__device__ inline void max3_after_mfma(f32x16& a, const f32x16& b, const f32x16& c) {
  SF_MAX3_4("s_nop 7\n\ts_nop 3\n\t", a, b, c, 0);
  SF_MAX3_4("", a, b, c, 4);
  SF_MAX3_4("", a, b, c, 8);
  SF_MAX3_4("", a, b, c, 12);
}
// The same on values that VALU or LDS instructions produced (no hazard of that kind).
__device__ inline float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

struct CprArgs {
  const u32x4* in;    // fp16 [B][H][W][CIN] as 16-byte pieces
  const u32x4* wpk;   // A operands [9][CIN/16][64]
  const float* bias;  // [32]
  uint16_t* out;      // fp16 [B][Ho][Wo][32]
  int B, H, W, Ho, Wo;
  int PC;             // pixels per LDS plane row: W/2 + 1
  int PB;             // bytes per LDS plane: (H + 2) * PC * pitch
  int n_seg;          // row segments of a frame (one wave each at a time)
  int row_pieces;     // 16-byte pieces per image row: W * CIN / 8
  int step_rows;      // image rows that the workgroup's threads cover at once: kNT / row_pieces
};

struct Rows {
  f32x16 e, o;  // accumulators of a convolution row: columns 2x and 2x+1
};

// CIN channels in; PPT 16-byte pieces per thread and frame; FPW frames per workgroup round.
template <int CIN, int PPT, int FPW>
__global__ __launch_bounds__(kNT, 2) void conv_pool_regs_kernel(CprArgs g) {
  constexpr int NS = CIN / 16, C8 = CIN / 8;
  constexpr int P = CIN == 16 ? 48 : 80;
  constexpr int LPR = 32 / FPW;  // lanes per pooled row
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (scalar: the row loops branch uniformly)
  const int j = lane & 31, lh = lane >> 5;
  const int fsel = j / LPR, xl = j % LPR;  // frame of the round and pooled column of this lane
  const int RPB = g.PC * P;                // bytes per LDS plane row
  const int FB = 2 * g.PB;                 // bytes per frame in LDS: even plane, odd plane

  // zeros once: the rings are never written again
  for (int i = tid; i < FPW * FB / 16; i += kNT) ((u32x4*)lds)[i] = u32x4{0u, 0u, 0u, 0u};
  // the filter bank behind the frames (the registers are needed for three accumulator sets)
  const u32x4* wl = (const u32x4*)(lds + FPW * FB) + lane;
  for (int i = tid; i < 9 * NS * 64; i += kNT) ((u32x4*)(lds + FPW * FB))[i] = g.wpk[i];
  // the bias in the accumulator layout: register 4*q4 + u holds channel 8*q4 + 4*lh + u
  f32x16 bias_acc;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 bv = *(const f32x4*)(g.bias + 8 * q4 + 4 * lh);
#pragma unroll
    for (int u = 0; u < 4; ++u) bias_acc[4 * q4 + u] = bv[u];
  }
  // The parameters have arrived before the first frame is requested (vmcnt(0), other counters
  // untouched).  Otherwise the compiler, which must assume their loads pending on some path,
  // drains the load counter ahead of every row loop that uses them, and that wait would catch
  // the next frame's pixels right after they have been requested.
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // The threads cover step_rows image rows at a time, one 16-byte piece each: thread tid has
  // piece tid % row_pieces (pixel x, channels 8*c8..) of row tid / row_pieces of the step.  In LDS:
  // plane x%2, row y + 1, plane column x/2 (even plane) or x/2 + 1 (odd plane: its column 0 is
  // image column -1).  Threads past step_rows * row_pieces idle.
  const int srow = tid / g.row_pieces, scol = tid - srow * g.row_pieces;
  const bool loader = srow < g.step_rows;
  const int pieces = g.H * g.row_pieces;
  int lds_off0;
  {
    const int px = scol / C8, c8 = scol - px * C8;
    lds_off0 = (px & 1) * g.PB + ((srow + 1) * g.PC + (px >> 1) + (px & 1)) * P + c8 * 16;
  }
  u32x4 nx[FPW][PPT];
  auto load_frames = [&](int b0) {
#pragma unroll
    for (int f = 0; f < FPW; ++f) {
      const u32x4* src = g.in + (size_t)min(b0 + f, g.B - 1) * pieces;  // (past the end: the last again)
#pragma unroll
      for (int k = 0; k < PPT; ++k) {
        // (an opaque move keeps the index from being computed ahead of the frame loop and spilled)
        int p = tid;
        asm volatile("" : "+v"(p));
        p += k * g.step_rows * g.row_pieces;
        nx[f][k] = src[loader && p < pieces ? p : pieces - 1];
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int f = 0; f < FPW; ++f)
#pragma unroll
      for (int k = 0; k < PPT; ++k)
        if (loader && srow + k * g.step_rows < g.H)
          *(u32x4*)(lds + f * FB + lds_off0 + k * g.step_rows * RPB) = nx[f][k];
  };

  const float ninf = -__builtin_inff();
  const bool live_x = xl < g.Wo;
  const int x = live_x ? xl : g.Wo - 1;
  const unsigned char* lane_base = lds + fsel * FB + x * P + lh * 16;
  // the lane that holds pooled column x-1 of the same frame and channels (column 0: itself,
  // which repeats O[0] in the maximum)
  const int left_lane = (xl == 0 ? lane : lane - 1) * 4;

  auto compute = [&](int b0) {
    const bool live = live_x && b0 + fsel < g.B;
    uint16_t* out_lane = g.out + ((size_t)min(b0 + fsel, g.B - 1) * g.Ho * g.Wo + x) * 32 + 4 * lh;
    // Accumulators of convolution row r (0 <= r < H): image rows r-1 .. r+1 = LDS rows r .. r+2.
    // 3 * NS steps (filter row, 16-channel group) of four pixel fragments, three weight
    // fragments and six MFMAs; a step's fragments are requested before the previous step's MFMAs
    // and no further ahead (the scheduling barriers: fragments of later steps would not fit the
    // registers beside three accumulator sets).
    struct Frag {
      u32x4 e0, e1, o0, o1, w0, w1, w2;
    };
    auto load_step = [&](int r, int t, Frag& f) {
      const int p = t / NS, sg = t % NS;
      const unsigned char* rowb = lane_base + (r + p) * RPB + sg * 32;
      f.e0 = *(const u32x4*)rowb;                 // image column 2x
      f.e1 = *(const u32x4*)(rowb + P);           // 2x+2
      f.o0 = *(const u32x4*)(rowb + g.PB);        // 2x-1
      f.o1 = *(const u32x4*)(rowb + g.PB + P);    // 2x+1
      f.w0 = wl[((p * 3 + 0) * NS + sg) * 64];
      f.w1 = wl[((p * 3 + 1) * NS + sg) * 64];
      f.w2 = wl[((p * 3 + 2) * NS + sg) * 64];
    };
    auto conv_row = [&](int r, Rows& a) {
      a.e = bias_acc;
      a.o = bias_acc;
      Frag f[2];
      load_step(r, 0, f[0]);
#pragma unroll
      for (int t = 0; t < 3 * NS; ++t) {
        if (t + 1 < 3 * NS) load_step(r, t + 1, f[(t + 1) & 1]);
        const Frag& c = f[t & 1];
        a.e = mfma(c.w0, c.o0, a.e);
        a.o = mfma(c.w0, c.e0, a.o);
        a.e = mfma(c.w1, c.e0, a.e);
        a.o = mfma(c.w1, c.o1, a.o);
        a.e = mfma(c.w2, c.o1, a.e);
        a.o = mfma(c.w2, c.e1, a.o);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // pooled row oy from the row maxima m: max(E[x], O[x], O[x-1]), rounded, stored
    auto emit = [&](int oy, const Rows& m) {
      uint16_t* dst = out_lane + (size_t)oy * g.Wo * 32;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float mo = m.o[4 * q4 + u];
          const float sh = __builtin_bit_cast(
              float, __builtin_amdgcn_ds_bpermute(left_lane, __builtin_bit_cast(int, mo)));
          v[u] = max3(m.e[4 * q4 + u], mo, sh);
        }
        const u32x2 ov = {pack_f16(v[0], v[1]), pack_f16(v[2], v[3])};
        if (live) *(u32x2*)(dst + 8 * q4) = ov;
      }
    };
    auto fill = [&](Rows& a) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        a.e[v] = ninf;
        a.o[v] = ninf;
      }
    };
    for (int seg = wave; seg < g.n_seg; seg += kNW) {
      const int oy0 = seg * g.Ho / g.n_seg, oy1 = (seg + 1) * g.Ho / g.n_seg;
      // Three accumulator sets take the roles carry (row 2y-1), row 2y, row 2y+1 in turn; the
      // maximum lands in the carry's set and the set of row 2y+1 is the next carry: two pooled
      // rows per trip, no copies.
      Rows a, b, c;
      if (oy0 > 0) conv_row(2 * oy0 - 1, a);
      else fill(a);  // row -1 is the pool's padding
      for (int oy = oy0; oy < oy1; oy += 2) {
        conv_row(2 * oy, b);
        if (2 * oy + 1 < g.H) conv_row(2 * oy + 1, c);
        else fill(c);  // (the last pooled row of an odd height)
        max3_after_mfma(a.e, b.e, c.e);
        max3_after_mfma(a.o, b.o, c.o);
        emit(oy, a);
        if (oy + 1 >= oy1) break;
        conv_row(2 * oy + 2, b);
        if (2 * oy + 3 < g.H) conv_row(2 * oy + 3, a);
        else fill(a);
        max3_after_mfma(c.e, b.e, a.e);
        max3_after_mfma(c.o, b.o, a.o);
        emit(oy + 1, c);
      }
    }
  };

  int b0 = blockIdx.x * FPW;
  load_frames(b0);
  __syncthreads();  // zeros in place
  for (; b0 < g.B; b0 += gridDim.x * FPW) {
    stage();
    __syncthreads();
    if (b0 + (int)gridDim.x * FPW < g.B) load_frames(b0 + (int)gridDim.x * FPW);
    compute(b0);
    __syncthreads();  // every read of these frames done before the next ones are staged
  }
}

int pitch_of(int cin) { return cin == 16 ? 48 : 80; }
size_t plane_bytes(int cin, int H, int W) { return (size_t)(H + 2) * (W / 2 + 1) * pitch_of(cin); }
int frames_per_round(int W) { return (W / 2) <= 16 ? 2 : 1; }
int step_rows_of(int cin, int W) { return kNT / (W * (cin / 8)); }
int pieces_per_thread(int cin, int H, int W) {
  const int sr = step_rows_of(cin, W);
  return (H + sr - 1) / sr;
}
size_t lds_bytes_of(int cin, int H, int W) {
  return 2 * plane_bytes(cin, H, W) * frames_per_round(W) + (size_t)9 * (cin / 16) * 1024;
}

template <int CIN, int PPT, int FPW>
hipError_t launch_t(const CprArgs& g, size_t lds_bytes, hipStream_t st) {
  auto kern = conv_pool_regs_kernel<CIN, PPT, FPW>;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&] {
    attr_status = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int rounds = (g.B + FPW - 1) / FPW;
  const int blocks = rounds < 256 ? rounds : 256;  // one workgroup per CU, each walking its share of the frames
  kern<<<blocks, kNT, lds_bytes, st>>>(g);
  return hipGetLastError();
}

template <int CIN>
hipError_t launch_c(const CprArgs& g, int ppt, int fpw, size_t lds_bytes, hipStream_t st) {
  if (fpw == 1) {
    if (ppt <= 3) return launch_t<CIN, 3, 1>(g, lds_bytes, st);
    if (ppt <= 6) return launch_t<CIN, 6, 1>(g, lds_bytes, st);
    return launch_t<CIN, 9, 1>(g, lds_bytes, st);
  }
  if (ppt <= 2) return launch_t<CIN, 2, 2>(g, lds_bytes, st);
  return launch_t<CIN, 5, 2>(g, lds_bytes, st);
}

}  // namespace

// 16 or 32 -> 32 channels; even frame width of at most 64 (pooled width at most 32); the frames of
// a round and the filter bank within 160 KB of LDS, and a frame within nine (one frame per round) or five
// (two frames) pieces per thread.
bool conv_pool_regs_supported(int cin, int cout, int H, int W) {
  if (!((cin == 16 || cin == 32) && cout == 32 && H >= 1 && W >= 2 && W % 2 == 0 && W <= 64)) return false;
  const int fpw = frames_per_round(W);
  return lds_bytes_of(cin, H, W) <= kMaxLds && pieces_per_thread(cin, H, W) <= (fpw == 1 ? 9 : 5);
}

// in: fp16 [B][H][W][cin]; wpk / bias32 as packed for the patch kernels with fp16 weights;
// out: fp16 [B][(H-1)/2+1][W/2][32].
hipError_t launch_conv_pool_regs(const void* in, const uint16_t* wpk, const float* bias32, void* out, int B,
                                 int H, int W, int cin, hipStream_t st) {
  if ((long long)B * H * W == 0) return hipSuccess;
  if (!conv_pool_regs_supported(cin, 32, H, W)) return hipErrorInvalidValue;
  CprArgs g;
  g.in = (const u32x4*)in; g.wpk = (const u32x4*)wpk; g.bias = bias32; g.out = (uint16_t*)out;
  g.B = B; g.H = H; g.W = W; g.Ho = (H - 1) / 2 + 1; g.Wo = W / 2;
  g.PC = W / 2 + 1;
  g.PB = (int)plane_bytes(cin, H, W);
  g.n_seg = g.Ho < kNW ? g.Ho : kNW;
  g.row_pieces = W * (cin / 8);
  g.step_rows = step_rows_of(cin, W);
  const int fpw = frames_per_round(W);
  const size_t lds_bytes = lds_bytes_of(cin, H, W);
  const int ppt = pieces_per_thread(cin, H, W);
  return cin == 16 ? launch_c<16>(g, ppt, fpw, lds_bytes, st) : launch_c<32>(g, ppt, fpw, lds_bytes, st);
}

}  // namespace sf

// Internal declarations of the sf_policy library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "sf_policy.h"

namespace sf {

// One convolution as executed.  Activations between layers are channels-last
// fp32 ([B][H][W][C]); only the observation is planar bytes.
struct ConvLayer {
  int cin, H, W;          // input
  int cout, k, s, pad;    // filter
  int Ho, Wo;             // output
  float* w_khwc_o;        // dev [k][k][cin][cout]
  float* bias;            // dev [cout]
  int relu_in, relu_out;  // ReLU applied to the input as it is read / to the result
  int add_residual;       // result += residual buffer before relu_out
  int impl;               // kernel choice, see ConvImpl
  int tile;               // tile configuration of the GEMM kernel, fixed at create
  float* wpk;             // dev, layout of the chosen MFMA kernel (or null)
  float* bpk;             // dev, bias as the chosen MFMA kernel wants it (or null)
  int* ipk;               // dev, int8 digit planes of the int8 first-convolution kernel
  float* spk;             // dev, per-channel scales of that kernel
  float* bpk8;            // dev, bias as that kernel wants it
  int planes;             // digit planes that kernel uses (2 or 3)
  uint16_t* wbf;          // dev, bf16 [Npad][Kpad] weights of the bf16 kernel
  float* bbf;             // dev, bias padded to Npad
  int Kpad;
  int in_f32, out_f32;    // bf16 kernel: element type of its input / output tensors
  float* w_cpqo;          // dev, fp32 [c][p][q][cout] for the byte-input 3x3 kernel
  uint16_t* wsp;          // dev, A operands in a second layout: of the register-pooled first convolution,
                          // or of a 16 -> 16 channel block convolution for the stage kernel (or null)
};
enum ConvImpl {
  CONV_GENERIC = 0, CONV1_U8_MFMA = 1, CONV_GEMM_MFMA = 2, CONV1_U8_I8 = 3,
  CONV_BF16 = 4,        // bf16 MFMA implicit GEMM, bf16 activations
  CONV3X3_U8_BF16 = 5,  // first convolution of the residual encoder, bytes in, 16-bit out (VALU)
  CONV3X3_PATCH = 6,    // 3x3/s1/p1 on the 16-bit MFMA with an LDS-staged input patch
  CONV3X3_STEM = 7,     // first convolution of the residual encoder on the 16-bit MFMA
  CONV3X3_POOL = 8,     // stage convolution fused with the max-pool behind it
  RES_BLOCK = 9,        // a whole residual block (this layer and the next) in one kernel
  RES_STAGE = 11,       // all residual blocks of a stage in one kernel, frame resident in LDS
  STEM_POOL = 12,       // first convolution of the residual encoder and its max-pool, pooled in registers
  CONV_POOL_REGS = 13,  // stage convolution (16 or 32 -> 32 channels) and its max-pool, pooled in registers
  CONV_IMAGE_BF16 = 10  // 16-bit MFMA with the frame's input image resident in LDS
};

// Kernel-selection switches (environment variables, for A/B measurements and for the tests
// that force a fallback kernel).  Read once, in sf_policy_create; a weight update replays the
// plan with the values stored in the policy.
struct Switches {
  bool force_generic = false;    // SF_FORCE_GENERIC: shape-agnostic kernels everywhere
  int conv1 = 0;                 // SF_CONV1: 0 = by the admission test of the fixed-point bank,
                                 // 1 = "fp32" (fp32 MFMA forced), 2 = "i8" (digit planes forced)
  int conv1_waves = 0;           // SF_CONV1_WAVES
  int gemm_tile = 0, fc_tile = 0, gru_bm = 0;  // SF_GEMM_TILE, SF_FC_TILE, SF_GRU_BM (0 = default)
  bool no_rnn_pairs = false;     // SF_NO_RNN_PAIRS
  bool no_bf16_path = false;     // SF_NO_BF16_PATH
  bool no_rnn_bf16 = false;      // SF_NO_RNN_BF16
  int conv_bf16_tc = 0;          // SF_CONV_BF16_TC
  bool no_conv1_image = false;   // SF_NO_CONV1_IMAGE
  bool no_conv_image = false;    // SF_NO_CONV_IMAGE
  bool no_conv12_fuse = false;   // SF_NO_CONV12_FUSE
  bool fc_out_f32 = false;       // SF_FC_OUT_F32
  bool no_patch_conv = false;    // SF_NO_PATCH_CONV
  bool no_fused_resnet = false;  // SF_NO_FUSED_RESNET
  bool no_res_stage = false;     // SF_NO_RES_STAGE
  bool no_stem_pool = false;     // SF_NO_STEM_POOL
  bool no_conv_pool_regs = false;  // SF_NO_CONV_POOL_REGS
  bool no_rnn_seq = false;         // SF_NO_RNN_SEQ
  bool act_bf16 = false;         // SF_ACT_BF16
  bool stream_f32 = false;       // SF_STREAM_F32
};

// One kernel launch of the step, fixed at create time.
enum OpKind { OP_CONV, OP_POOL, OP_FC, OP_MEAS, OP_GRU, OP_HEADS };
struct Op {
  OpKind kind;
  std::string name;
  int64_t flops_per_row;  // 2 per multiply-add
  int conv;               // index into Policy::convs (OP_CONV); measurement layer, or -1 = all
                          // layers in one launch (OP_MEAS); else -1
  int in_buf, out_buf;    // activation buffer indices; in_buf -1 = the observation
  int resid_buf;          // buffer added to the result, or -1
  int C, H, W;            // OP_POOL: input shape
  int n_sub = 0;          // RES_STAGE: convolutions covered (2 per block)
  int mid_buf = -1;       // first and second convolution in one launch: buffer for the first
                          // layer's output when the two have to run separately after all
};

struct Policy {
  sf_policy_config cfg;
  Switches sw;
  int device;
  int flat;   // encoder output elements per row
  int sumA;   // total logits per row
  int max_head = 0;  // categories of the largest head
  std::vector<ConvLayer> convs;  // in execution order
  // packed weights
  float* fc_w_t;      // dev [flat (channels-last order)][fc_dim]
  float* fc_b;        // dev [fc_dim]
  float* fc_wt;       // dev [fc_dim][flat (channels-last order)] for the MFMA GEMM, or null
  uint16_t* fc_wbf;   // dev bf16 [fc_dim pad 32][flat pad 64] for the bf16 kernel, or null
  float* fc_bbf;
  int fc_Kpad;
  bool bf16_path;     // encoder and FC run on the 16-bit MFMA kernels with 16-bit activations
  bool act_f16;       // ... whose activation element type is fp16 instead of bf16
  bool stream_f32;    // residual encoder: the residual stream is stored in fp32
  int fc_tile;
  // recurrent core (GRU: G = 3 gate blocks, LSTM: G = 4); core input = fc_dim + meas_out_dim
  float* gru_wih_t;   // dev [core input][G*H]
  float* gru_whh_t;   // dev [H][G*H]
  float* gru_wih;     // dev [G*H][core input] (canonical) for the MFMA kernel, or null
  float* gru_whh;     // dev [G*H][H]
  float* rnn_seq_w = nullptr;  // dev: both matrices in the operand order of k_rnn_seq.hip, or null
  int gru_bm;         // rows per workgroup of the MFMA kernel, fixed at create
  double conv1_ratio2 = 0, conv1_ratio3 = 0;  // admission test of the first convolution's digit planes
  int conv1_image = 1;      // first convolution: frame-resident variant where it applies
  int fc_out_bf16 = 0;      // the FC kernel hands bf16 values to the 16-bit recurrent kernel
  int conv_bf16_tc = 0;     // 16-bit conv kernel: 0 = channel blocks per workgroup by grid size, 1 / 2 forced
  int rnn_plain_loops = 1;  // GRU on the MFMA: the two-plain-loops form where the chunk counts allow it
  uint16_t* rnn_wih_bf;  // dev bf16 [G*H][core input] for the 16-bit MFMA kernel, or null
  uint16_t* rnn_whh_bf;  // dev bf16 [G*H][H]
  float* gru_bih;     // dev [G*H]
  float* gru_bhh;     // dev [G*H]
  int state_dim;      // floats per state row: H (GRU) or 2H (LSTM: [h | c])
  // measurement encoder of the full architecture (n_meas = 0: none)
  int n_meas;
  int meas_out_dim;
  int meas_in_dim[SF_MAX_MEAS_LAYERS];
  float* meas_w_t[SF_MAX_MEAS_LAYERS];  // dev [in][out]
  float* meas_b[SF_MAX_MEAS_LAYERS];
  float* meas_buf[SF_MAX_MEAS_LAYERS];  // dev [max_batch][meas_hidden[l]]
  float* head_w;      // dev [sumA + 1][H]   (last row: value head)
  float* head_b;      // dev [sumA + 1]
  int32_t* head_off;  // dev [n_heads + 1]   prefix sums of head_sizes
  // workspace, sized for max_batch
  float* act[3];      // three activation buffers of act_elems floats per row
  size_t act_elems;
  float* fc_out;      // dev [max_batch][fc_dim]
  float* h_new;       // dev [max_batch][state_dim]: new states of an indexed step before the scatter
  float* trash;       // dev, 64 floats: target of stores that fall outside a tensor
  std::vector<void*> allocations;
  std::vector<size_t> alloc_bytes;   // size of each allocation, in allocation order
  size_t upload_bytes = 0;           // bytes of packed weights uploaded at create (+ alignment slack)
  // weight updates: page-locked staging area for the packed weights and the event that
  // marks the end of the last update's copies out of it
  unsigned char* stage = nullptr;
  size_t stage_bytes = 0;
  hipEvent_t stage_ev = nullptr;
  int64_t flops_per_row;
  std::vector<Op> ops;    // the launch sequence
  int enc_buf;            // buffer holding the encoder output
  int conv1_waves = 0;    // wavefronts for the first-convolution kernel (0 = default)
  // optional per-launch timing (measurement aid)
  bool timing = false;
  std::vector<hipEvent_t> events;  // ops.size() + 1
};

void set_error(const char* fmt, ...);

// ---- generic kernels (any shape) ----
hipError_t launch_conv_generic(const ConvLayer& L, int B, const void* in, bool in_is_u8_planar,
                               float obs_sub, float obs_mul, const float* residual, float* out,
                               hipStream_t st);
hipError_t launch_maxpool3x3s2p1(int B, int C, int H, int W, const float* in, float* out,
                                 hipStream_t st);
hipError_t launch_linear_generic(int B, int n_in, int n_out, const float* in, const float* w_t,
                                 const float* bias, int relu, float* out, hipStream_t st);
bool meas_mlp_supported(int n0, int n1);
hipError_t launch_meas_mlp(int B, int n0, const float* meas, const float* w1_t, const float* b1, int n1,
                           const float* w2_t, const float* b2, int n2, float* out, hipStream_t st);
hipError_t launch_rnn_generic(int lstm, int B, int n1, int n2, int H, const float* x1, const float* x2,
                              const float* h_in, const uint8_t* done, const float* wih_t,
                              const float* whh_t, const float* bih, const float* bhh, float* h_out,
                              const int32_t* ids, int n_env, hipStream_t st);
hipError_t launch_heads(int B, int H, int n_heads, int sumA, const int32_t* head_off,
                        const float* h, const float* head_w, const float* head_b, uint64_t seed,
                        uint64_t step, int32_t* actions, float* logp, float* value,
                        float* logits_opt, const int32_t* ids, float* h_table, int n_env,
                        int state_dim, int max_head, hipStream_t st);

hipError_t launch_copy16(const void* src, void* dst, long long bytes, hipStream_t st);

// ---- MFMA kernels (specialised shapes) ----
bool conv1_mfma_supported(const ConvLayer& L);
void conv1_mfma_pack(const float* w, const float* bias, int cin, float obs_sub, float obs_mul,
                     std::vector<float>& wpk, std::vector<float>& bpk);
hipError_t launch_conv1_mfma(const ConvLayer& L, int B, const uint8_t* obs, const float* wpk,
                             const float* bpk, float* out, float* trash, int waves_hint,
                             float obs_sub, hipStream_t st);

bool conv1_i8_supported(const ConvLayer& L);
// Result of the admission test of a fixed-point filter bank: worst channel's ratio of the
// bank's error bound to that of the floating-point path it replaces, with two and with
// three digit planes (<= 1: admitted).
struct Conv1I8Info {
  double ratio2, ratio3;
};
void conv1_i8_pack(const float* w, const float* bias, int cin, float obs_sub, float obs_mul,
                   bool bf16_weights, std::vector<int>& wpk, std::vector<float>& scale,
                   std::vector<float>& bpk, Conv1I8Info* info);
hipError_t launch_conv1_i8(const ConvLayer& L, int B, const uint8_t* obs, const int* wpk,
                           const float* scale, const float* bpk, void* out, int out_bf16,
                           int planes, int waves_hint, int image, hipStream_t st);
bool conv_bf16_supported(int Cin, int N);
void conv_bf16_pack(const float* w, const float* bias, int cout, int cin, int k, bool f16,
                    std::vector<uint16_t>& wt, std::vector<float>& b, int* Kpad);
hipError_t launch_conv_bf16(const void* in, const uint16_t* wt, const float* bias,
                            const void* resid, void* out, int B, int H, int W, int Cin, int ks,
                            int stride, int pad, int Ho, int Wo, int N, int Kpad, int relu_in,
                            int relu_out, int in_f32, int resid_f32, int out_f32, int f16,
                            int tc_force, int tag, hipStream_t st);
hipError_t launch_maxpool_bf16(int B, int C, int H, int W, const void* in, void* out, int out_f32,
                               int f16, hipStream_t st);
bool conv3x3_u8_bf16_supported(int cout);
hipError_t launch_conv3x3_u8_bf16(int B, int Cin, int H, int W, int cout, const uint8_t* obs,
                                  const float* w_cpqo, const float* bias, void* out, float obs_sub,
                                  float obs_mul, int f16, hipStream_t st);
bool conv3x3_patch_supported(int cin, int cout, int k, int stride, int pad);
void conv3x3_patch_pack(const float* w, const float* bias, int cout, int cin, bool f16,
                        std::vector<uint16_t>& wpk, std::vector<float>& b32);
hipError_t launch_conv3x3_patch(const void* in, const uint16_t* wpk, const float* bias32,
                                const void* resid, int resid_f32, void* out, int B, int H, int W,
                                int cin, int cout, int in_f32, int relu_in, int relu_out,
                                int out_f32, int f16, hipStream_t st);
bool conv3x3_pool_supported(int cin, int cout, int W);
hipError_t launch_conv3x3_pool(const void* in, const uint16_t* wpk, const float* bias32, void* out,
                               int B, int H, int W, int cin, int cout, float obs_sub, float obs_mul,
                               hipStream_t st);
bool res_block_supported(int c);
hipError_t launch_res_block(const void* x, const uint16_t* wa, const float* ba, const uint16_t* wb,
                            const float* bb, void* out, int B, int H, int W, int c, int relu_out,
                            hipStream_t st);
bool res_stage_supported(int c, int H, int W, int n_blocks);
void res_stage_pack16(const float* w, bool f16, std::vector<uint16_t>& wpk);
hipError_t launch_res_stage(const void* x, void* out, const uint16_t* const* wpk, const float* const* bias,
                            int n_convs, int B, int H, int W, int c, int relu_out, hipStream_t st);
uint16_t conv_weight_bits(float v, bool f16);
bool stem_pool_supported(int cin, int cout, int H, int W);
void stem_pool_pack(const float* w, bool f16, std::vector<uint16_t>& wpk);
hipError_t launch_stem_pool(const uint8_t* obs, const uint16_t* wpk, const float* bias, void* out, int B,
                            int H, int W, float obs_sub, float obs_mul, hipStream_t st);
bool conv_pool_regs_supported(int cin, int cout, int H, int W);
hipError_t launch_conv_pool_regs(const void* in, const uint16_t* wpk, const float* bias32, void* out, int B,
                                 int H, int W, int cin, hipStream_t st);
bool conv3x3_stem_supported(int cin, int cout);
void conv3x3_stem_pack(const float* w, const float* bias, int cout, bool f16,
                       std::vector<uint16_t>& wpk, std::vector<float>& b32);
hipError_t launch_conv3x3_stem(const uint8_t* obs, const uint16_t* wpk, const float* bias32, void* out,
                               int B, int H, int W, int cout, float obs_sub, float obs_mul, int f16,
                               hipStream_t st);
bool rnn_mfma_supported(int I1, int I2, int H);
hipError_t launch_rnn_mfma(int lstm, int B, int I1, int I2, int H, const float* x1, const float* x2,
                           const float* h_in, const uint8_t* done, const float* w_ih,
                           const float* w_hh, const float* b_ih, const float* b_hh, float* h_out,
                           int bm, int plain_loops, const int32_t* ids, int n_env, hipStream_t st);
int rnn_mfma_pick_bm(int max_batch, int H);
// the cell for the few rows per time step of the pass over trajectories (k_rnn_seq.hip)
bool rnn_seq_supported(int I1, int I2, int H);
void rnn_seq_pack(const float* w_ih, const float* w_hh, int I, int H, int lstm, std::vector<float>& out);
hipError_t launch_rnn_seq(int lstm, int B, int I1, int I2, int H, const void* x1, int x1_bf16, const float* x2,
                          const float* h_in, const uint8_t* done, const float* wpk, const float* b_ih,
                          const float* b_hh, float* h_out, hipStream_t st);
bool rnn_bf16_supported(int I1, int I2, int H);
void rnn_bf16_pack(const float* w, size_t n, std::vector<uint16_t>& out);
hipError_t launch_rnn_bf16(int lstm, int B, int I1, int I2, int H, const void* x1, int x1_bf16,
                           const float* x2, const float* h_in, const uint8_t* done,
                           const uint16_t* w_ih, const uint16_t* w_hh, const float* b_ih,
                           const float* b_hh, float* h_out, const int32_t* ids, int n_env,
                           hipStream_t st);
bool conv_image_bf16_supported(int Cin, int ksize, int stride, int pad, int H, int W, int Ho, int Wo,
                               int N);
void conv_image_bf16_pack(const float* w, int cout, int cin, int k, std::vector<uint16_t>& wpk);
hipError_t launch_conv_image_bf16(const void* in, const uint16_t* wpk, const float* bias, void* out,
                                  int B, int H, int W, int Cin, int ksize, int stride, int Ho,
                                  int Wo, int N, int relu, hipStream_t st);
bool conv12_fused_bf16_supported(int cin, int H, int W, const sf_conv& c1, const sf_conv& c2);
hipError_t launch_conv12_fused_bf16(const ConvLayer& L1, const ConvLayer& L2, int B, const uint8_t* obs,
                                    void* out, hipStream_t st);
bool gemm_mfma_supported(int Cin, int ksize, int pad, int N);
int gemm_mfma_pick_tile(long long M, int N, int K, int seg_len);
hipError_t launch_gemm_mfma(const float* A, const float* Wt, const float* bias, float* out, int B,
                            int H, int W, int Cin, int ksize, int stride, int Ho, int Wo, int N,
                            int relu, int tile, int tag, hipStream_t st);

}  // namespace sf

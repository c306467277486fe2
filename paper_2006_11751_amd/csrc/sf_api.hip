// C ABI of the sf_policy library: validation, weight packing, workspace and the
// launch sequence of one policy step (see include/sf_policy.h for the contract).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "sf_internal.h"

namespace sf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

namespace {

// Round to the nearest bf16 (ties to even) and widen again.
float bf16_round(float v) {
  uint32_t u;
  memcpy(&u, &v, 4);
  if ((u & 0x7F800000u) != 0x7F800000u) u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
  memcpy(&v, &u, 4);
  return v;
}

// Allocates and fills the device buffers of a policy.  In replay mode (a weight update)
// nothing is allocated: the k-th request returns the k-th buffer of `target`, whose size
// must match, and an upload only writes the packed values into `target`'s page-locked
// staging area and notes the copy; flush() enqueues the noted copies once the whole plan has
// been packed and checked, so that a failure on the way leaves the live weights untouched.
struct Builder {
  Policy* p;
  bool bf16;
  int status = SF_OK;
  Policy* target = nullptr;  // replay: the live policy whose buffers are refilled
  size_t next = 0, stage_off = 0;
  struct Copy {
    void* dst;
    size_t off, bytes;
  };
  std::vector<Copy> copies;

  int flush(hipStream_t stream) {
    for (const Copy& c : copies) {
      hipError_t e = hipMemcpyAsync(c.dst, target->stage + c.off, c.bytes, hipMemcpyHostToDevice, stream);
      if (e != hipSuccess) {
        set_error("weight update: hipMemcpyAsync failed: %s", hipGetErrorString(e));
        return SF_ERR_DEVICE;
      }
    }
    return SF_OK;
  }

  void* dev_alloc(size_t bytes) {
    if (bytes == 0) bytes = 4;
    if (target) {
      if (next >= target->allocations.size() || target->alloc_bytes[next] != bytes) {
        if (status == SF_OK) {
          set_error("weight update: buffer %zu does not match the policy built at create", next);
          status = SF_ERR_SHAPE;
        }
        return nullptr;
      }
      return target->allocations[next++];
    }
    void* d = nullptr;
    hipError_t e = hipMalloc(&d, bytes);
    if (e != hipSuccess) {
      set_error("hipMalloc(%zu bytes) failed: %s", bytes, hipGetErrorString(e));
      status = SF_ERR_OOM;
      return nullptr;
    }
    p->allocations.push_back(d);
    p->alloc_bytes.push_back(bytes);
    return d;
  }

  template <typename T>
  T* upload(const std::vector<T>& host) {
    T* d = (T*)dev_alloc(host.size() * sizeof(T));
    if (!d) return nullptr;
    const size_t n = host.size() * sizeof(T);
    if (target) {
      const size_t off = (stage_off + 15) & ~(size_t)15;
      if (off + n > target->stage_bytes) {
        if (status == SF_OK) {
          set_error("weight update: staging area too small");
          status = SF_ERR_SHAPE;
        }
        return nullptr;
      }
      memcpy(target->stage + off, host.data(), n);
      stage_off = off + n;
      copies.push_back(Copy{d, off, n});
      return d;
    }
    p->upload_bytes += n + 16;
    hipError_t e = hipMemcpy(d, host.data(), n, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      set_error("hipMemcpy to device failed: %s", hipGetErrorString(e));
      status = SF_ERR_DEVICE;
      return nullptr;
    }
    return d;
  }

  float q(float v) const { return bf16 ? bf16_round(v) : v; }

  // [cout][cin][k][k] -> [k][k][cin][cout]
  float* pack_conv(const float* w, int cout, int cin, int k) {
    std::vector<float> t((size_t)cout * cin * k * k);
    for (int o = 0; o < cout; ++o)
      for (int c = 0; c < cin; ++c)
        for (int a = 0; a < k; ++a)
          for (int b = 0; b < k; ++b)
            t[(((size_t)a * k + b) * cin + c) * cout + o] =
                q(w[(((size_t)o * cin + c) * k + a) * k + b]);
    return upload(t);
  }

  float* pack_vec(const float* v, size_t n) {
    std::vector<float> t(n);
    for (size_t i = 0; i < n; ++i) t[i] = q(v[i]);
    return upload(t);
  }

  // [n_out][n_in] -> [n_in][n_out]
  float* pack_transposed(const float* w, int n_out, int n_in) {
    std::vector<float> t((size_t)n_out * n_in);
    for (int o = 0; o < n_out; ++o)
      for (int i = 0; i < n_in; ++i) t[(size_t)i * n_out + o] = q(w[(size_t)o * n_in + i]);
    return upload(t);
  }
};

int check_config(const sf_policy_config* c, int* Cf, int* Hf, int* Wf) {
  if (c->max_batch < 1 || c->max_batch > 65535) {
    set_error("max_batch %d outside [1, 65535]", c->max_batch);
    return SF_ERR_SHAPE;
  }
  if (c->obs_c < 1 || c->obs_h < 1 || c->obs_w < 1) {
    set_error("empty observation shape");
    return SF_ERR_SHAPE;
  }
  int C = c->obs_c, H = c->obs_h, W = c->obs_w;
  if (c->encoder == SF_ENCODER_CONV) {
    if (c->n_conv < 1 || c->n_conv > SF_MAX_CONV) {
      set_error("n_conv %d outside [1, %d]", c->n_conv, SF_MAX_CONV);
      return SF_ERR_SHAPE;
    }
    for (int l = 0; l < c->n_conv; ++l) {
      const sf_conv& v = c->conv[l];
      if (v.cout < 1 || v.k < 1 || v.stride < 1 || v.pad < 0 || H + 2 * v.pad < v.k ||
          W + 2 * v.pad < v.k) {
        set_error("convolution %d has an empty output or bad parameters", l);
        return SF_ERR_SHAPE;
      }
      H = (H + 2 * v.pad - v.k) / v.stride + 1;
      W = (W + 2 * v.pad - v.k) / v.stride + 1;
      C = v.cout;
    }
  } else if (c->encoder == SF_ENCODER_RESNET) {
    if (c->n_stage < 1 || c->n_stage > SF_MAX_STAGE || c->blocks_per_stage < 0 ||
        c->n_stage * (1 + 2 * c->blocks_per_stage) > SF_MAX_CONV_TENSORS) {
      set_error("bad residual encoder description");
      return SF_ERR_SHAPE;
    }
    for (int s = 0; s < c->n_stage; ++s) {
      if (c->stage_ch[s] < 1) {
        set_error("stage %d has no channels", s);
        return SF_ERR_SHAPE;
      }
      C = c->stage_ch[s];
      H = (H - 1) / 2 + 1;
      W = (W - 1) / 2 + 1;
    }
  } else {
    set_error("unknown encoder %d", c->encoder);
    return SF_ERR_SHAPE;
  }
  if (c->fc_dim < 1 || c->rnn_dim < 1) {
    set_error("fc_dim and rnn_dim must be positive");
    return SF_ERR_SHAPE;
  }
  if (c->n_heads < 1 || c->n_heads > SF_MAX_HEADS) {
    set_error("n_heads %d outside [1, %d]", c->n_heads, SF_MAX_HEADS);
    return SF_ERR_SHAPE;
  }
  int sumA = 0;
  for (int k = 0; k < c->n_heads; ++k) {
    if (c->head_sizes[k] < 1 || c->head_sizes[k] > 65535) {
      set_error("head %d has size %d", k, c->head_sizes[k]);
      return SF_ERR_SHAPE;
    }
    sumA += c->head_sizes[k];
  }
  if (sumA + 1 > 1024) {
    set_error("more than 1023 logits per row");
    return SF_ERR_SHAPE;
  }
  if (c->dtype != SF_DTYPE_FP32 && c->dtype != SF_DTYPE_BF16) {
    set_error("unknown dtype %d", c->dtype);
    return SF_ERR_SHAPE;
  }
  if (c->rnn_type != SF_RNN_GRU && c->rnn_type != SF_RNN_LSTM) {
    set_error("unknown rnn_type %d", c->rnn_type);
    return SF_ERR_SHAPE;
  }
  if (c->meas_dim < 0 || c->meas_dim > 65535) {
    set_error("meas_dim %d outside [0, 65535]", c->meas_dim);
    return SF_ERR_SHAPE;
  }
  if (c->meas_dim > 0) {
    if (c->n_meas_layers < 1 || c->n_meas_layers > SF_MAX_MEAS_LAYERS) {
      set_error("n_meas_layers %d outside [1, %d]", c->n_meas_layers, SF_MAX_MEAS_LAYERS);
      return SF_ERR_SHAPE;
    }
    for (int l = 0; l < c->n_meas_layers; ++l)
      if (c->meas_hidden[l] < 1 || c->meas_hidden[l] > 65535) {
        set_error("measurement layer %d has width %d", l, c->meas_hidden[l]);
        return SF_ERR_SHAPE;
      }
  }
  *Cf = C;
  *Hf = H;
  *Wf = W;
  return SF_OK;
}

bool env_set(const char* name) { return getenv(name) != nullptr; }
int env_int(const char* name) {
  const char* v = getenv(name);
  return v ? atoi(v) : 0;
}

// The only place the environment is read.
Switches read_switches() {
  Switches sw;
  sw.force_generic = env_set("SF_FORCE_GENERIC");
  const char* c1 = getenv("SF_CONV1");
  sw.conv1 = !c1 ? 0 : (!strcmp(c1, "fp32") ? 1 : (!strcmp(c1, "i8") ? 2 : 0));
  sw.conv1_waves = env_int("SF_CONV1_WAVES");
  sw.gemm_tile = env_int("SF_GEMM_TILE");
  sw.fc_tile = env_int("SF_FC_TILE");
  sw.gru_bm = env_int("SF_GRU_BM");
  sw.no_rnn_pairs = env_set("SF_NO_RNN_PAIRS");
  sw.no_bf16_path = env_set("SF_NO_BF16_PATH");
  sw.no_rnn_bf16 = env_set("SF_NO_RNN_BF16");
  sw.conv_bf16_tc = env_int("SF_CONV_BF16_TC");
  sw.no_conv1_image = env_set("SF_NO_CONV1_IMAGE");
  sw.no_conv_image = env_set("SF_NO_CONV_IMAGE");
  sw.no_conv12_fuse = env_set("SF_NO_CONV12_FUSE");
  sw.fc_out_f32 = env_set("SF_FC_OUT_F32");
  sw.no_patch_conv = env_set("SF_NO_PATCH_CONV");
  sw.no_fused_resnet = env_set("SF_NO_FUSED_RESNET");
  sw.no_res_stage = env_set("SF_NO_RES_STAGE");
  sw.no_stem_pool = env_set("SF_NO_STEM_POOL");
  sw.no_conv_pool_regs = env_set("SF_NO_CONV_POOL_REGS");
  sw.no_rnn_seq = env_set("SF_NO_RNN_SEQ");
  sw.act_bf16 = env_set("SF_ACT_BF16");
  sw.stream_f32 = env_set("SF_STREAM_F32");
  return sw;
}

void free_policy(Policy* p) {
  if (!p) return;
  for (void* d : p->allocations) (void)hipFree(d);
  for (hipEvent_t ev : p->events)
    if (ev) (void)hipEventDestroy(ev);
  if (p->stage_ev) (void)hipEventDestroy(p->stage_ev);
  if (p->stage) (void)hipHostFree(p->stage);
  delete p;
}

}  // namespace
}  // namespace sf

using namespace sf;

namespace {

// Chooses the kernels, packs the weights and sizes the workspace of `p` for `cfg` under the
// switches in p->sw.  Shared by create (bld allocates) and by a weight update (bld replays into
// the live policy's buffers; `p` is then a scratch object whose plan and pointers come out
// identical).  The sequence of buffer requests depends on the description and the switches
// only, never on the parameter values.
int build_policy(Policy* p, const sf_policy_config* cfg, const sf_policy_weights* w, Builder& bld,
                 int Cf, int Hf, int Wf) {
  const Switches& sw = p->sw;
  p->cfg = *cfg;
  p->flat = Cf * Hf * Wf;
  p->conv1_waves = sw.conv1_waves;
  p->conv_bf16_tc = sw.conv_bf16_tc;
  p->conv1_image = sw.no_conv1_image ? 0 : 1;

  // bf16 configurations run the encoder and the FC layer on the bf16 kernels with bf16
  // activations, provided every layer has a shape those kernels take; otherwise the
  // fp32 kernels run on the (bf16-rounded) weights.
  p->bf16_path = false;
  if (cfg->dtype == SF_DTYPE_BF16 && !sw.force_generic && !sw.no_bf16_path) {
    bool ok = (p->flat % 8) == 0 && (cfg->fc_dim % 4) == 0;
    if (cfg->encoder == SF_ENCODER_CONV) {
      ConvLayer L0{};
      L0.cin = cfg->obs_c; L0.W = cfg->obs_w; L0.k = cfg->conv[0].k; L0.s = cfg->conv[0].stride;
      L0.pad = cfg->conv[0].pad; L0.cout = cfg->conv[0].cout; L0.relu_out = 1;
      ok = ok && conv1_i8_supported(L0);
      for (int l = 1; l < cfg->n_conv; ++l)
        ok = ok && conv_bf16_supported(cfg->conv[l - 1].cout, cfg->conv[l].cout);
    } else {
      ok = ok && conv3x3_u8_bf16_supported(cfg->stage_ch[0]);
      for (int s = 0; s < cfg->n_stage; ++s) {
        ok = ok && (cfg->stage_ch[s] % 8) == 0;
        if (s > 0) ok = ok && conv_bf16_supported(cfg->stage_ch[s - 1], cfg->stage_ch[s]);
      }
    }
    p->bf16_path = ok;
  }
  // The residual encoder is 15 convolutions deep: with 8-bit significands the rounding of
  // the activations alone exceeds the 2e-2 tolerance in the tails, so its 16-bit
  // activations are fp16 (the weights stay bf16 values, exactly representable in fp16).
  p->act_f16 = p->bf16_path && cfg->encoder == SF_ENCODER_RESNET && !sw.act_bf16;
  // With bf16 activations the residual stream is kept in fp32 so that its rounding does not
  // accumulate over the blocks; with fp16 activations that is not needed.
  p->stream_f32 = p->bf16_path && cfg->encoder == SF_ENCODER_RESNET &&
                  (!p->act_f16 || sw.stream_f32);

  // ---- encoder plan ----
  size_t act_elems = 0;
  int64_t macs = 0;
  {
    int C = cfg->obs_c, H = cfg->obs_h, W = cfg->obs_w;
    int ti = 0;
    auto add_conv = [&](const char* name, int cout, int k, int s, int pad, int relu_in,
                        int relu_out, int in_buf, int out_buf, int resid_buf) {
      ConvLayer L{};
      L.cin = C; L.H = H; L.W = W;
      L.cout = cout; L.k = k; L.s = s; L.pad = pad;
      L.Ho = (H + 2 * pad - k) / s + 1;
      L.Wo = (W + 2 * pad - k) / s + 1;
      L.w_khwc_o = nullptr;  // packed below if the shape-agnostic kernel runs this layer
      L.bias = bld.pack_vec(w->conv_b[ti], cout);
      // the bias as the configuration defines it (rounded to bf16 in a bf16 configuration),
      // for the packers that keep their own copy
      std::vector<float> qb(cout);
      for (int o = 0; o < cout; ++o) qb[o] = bld.q(w->conv_b[ti][o]);
      L.relu_in = relu_in; L.relu_out = relu_out; L.add_residual = resid_buf >= 0;
      L.impl = CONV_GENERIC;
      const bool allow_mfma = !sw.force_generic && !p->bf16_path;
      if (p->bf16_path) {
        if (in_buf >= 0) {
          std::vector<uint16_t> wt;
          std::vector<float> bb;
          conv_bf16_pack(w->conv_w[ti], qb.data(), cout, C, k, p->act_f16, wt, bb, &L.Kpad);
          L.wbf = bld.upload(wt);
          L.bbf = bld.upload(bb);
          L.impl = CONV_BF16;
          if (cfg->encoder == SF_ENCODER_RESNET && conv3x3_patch_supported(C, cout, k, s, pad) &&
              !sw.no_patch_conv) {
            conv3x3_patch_pack(w->conv_w[ti], qb.data(), cout, C, p->act_f16, wt, bb);
            L.wbf = bld.upload(wt);
            L.bbf = bld.upload(bb);
            L.impl = CONV3X3_PATCH;
            if (C == 16 && cout == 16 && p->act_f16) {
              // (block convolutions of a 16-channel stage: the stage kernel's tap-pair layout)
              std::vector<uint16_t> w16;
              res_stage_pack16(w->conv_w[ti], true, w16);
              L.wsp = bld.upload(w16);
            }
          }
          // Residual encoder: the stream x (pool outputs, block outputs) stays fp32 so that
          // its rounding does not accumulate over the blocks; branch intermediates and
          // stage-convolution outputs are bf16.  Plain stack: everything bf16.
          const bool resnet = p->stream_f32;
          L.in_f32 = resnet && !(relu_in == 0 && resid_buf >= 0);  // conv_b reads the bf16 branch
          L.out_f32 = resnet && resid_buf >= 0;
          if (cfg->encoder == SF_ENCODER_CONV && !p->act_f16 && !relu_in && resid_buf < 0 &&
              !sw.no_conv_image &&
              conv_image_bf16_supported(C, k, s, pad, H, W, L.Ho, L.Wo, cout)) {
            conv_image_bf16_pack(w->conv_w[ti], cout, C, k, wt);
            L.wbf = bld.upload(wt);
            L.impl = CONV_IMAGE_BF16;
          }
        } else if (cfg->encoder == SF_ENCODER_CONV) {
          // bf16 parameters carry 8 significant bits: two digit planes as a rule, the third
          // where the admission test asks for it
          std::vector<int> ipk;
          std::vector<float> spk, bpk;
          Conv1I8Info info;
          conv1_i8_pack(w->conv_w[ti], w->conv_b[ti], C, cfg->obs_sub, cfg->obs_mul, true, ipk, spk, bpk,
                        &info);
          L.ipk = bld.upload(ipk);
          L.spk = bld.upload(spk);
          L.bpk8 = bld.upload(bpk);
          L.impl = CONV1_U8_I8;
          L.planes = (sw.conv1 == 2 || info.ratio2 <= 1.0) ? 2 : 3;
          p->conv1_ratio2 = info.ratio2;
          p->conv1_ratio3 = info.ratio3;
        } else {
          std::vector<float> t((size_t)C * 9 * cout);  // [c][p][q][cout]
          for (int o = 0; o < cout; ++o)
            for (int c2 = 0; c2 < C; ++c2)
              for (int a = 0; a < 3; ++a)
                for (int b2 = 0; b2 < 3; ++b2)
                  t[(((size_t)c2 * 3 + a) * 3 + b2) * cout + o] =
                      bld.q(w->conv_w[ti][(((size_t)o * C + c2) * 3 + a) * 3 + b2]);
          L.w_cpqo = bld.upload(t);
          L.impl = CONV3X3_U8_BF16;
          if (conv3x3_stem_supported(C, cout) && !sw.no_patch_conv) {
            std::vector<uint16_t> wt;
            std::vector<float> bb;
            conv3x3_stem_pack(w->conv_w[ti], qb.data(), cout, p->act_f16, wt, bb);
            L.wbf = bld.upload(wt);
            L.bbf = bld.upload(bb);
            L.impl = CONV3X3_STEM;
            if (p->act_f16 && !sw.no_stem_pool && stem_pool_supported(C, cout, H, W)) {
              std::vector<uint16_t> ws;
              stem_pool_pack(w->conv_w[ti], true, ws);
              L.wsp = bld.upload(ws);
            }
          }
        }
      }
      if (in_buf >= 0 && allow_mfma && !relu_in && resid_buf < 0 &&
          gemm_mfma_supported(C, k, pad, cout)) {
        // [cout][cin][k][k] -> [cout][k][k][cin]: K ordered (filter row, filter column, channel)
        std::vector<float> t((size_t)cout * C * k * k);
        for (int o = 0; o < cout; ++o)
          for (int c2 = 0; c2 < C; ++c2)
            for (int a = 0; a < k; ++a)
              for (int b2 = 0; b2 < k; ++b2)
                t[(((size_t)o * k + a) * k + b2) * C + c2] =
                    bld.q(w->conv_w[ti][(((size_t)o * C + c2) * k + a) * k + b2]);
        L.wpk = bld.upload(t);
        L.bpk = L.bias;
        L.impl = CONV_GEMM_MFMA;
        L.tile = sw.gemm_tile > 0 ? sw.gemm_tile
                                  : gemm_mfma_pick_tile((long long)cfg->max_batch * L.Ho * L.Wo, cout,
                                                        k * k * C, k * C);
      }
      if (in_buf < 0 && allow_mfma && conv1_i8_supported(L) && conv1_mfma_supported(L)) {
        // First convolution of an fp32 network: three int8 digit planes of the folded filter
        // bank where that fixed-point image passes its admission test, the fp32 MFMA kernel
        // otherwise.  Both banks are packed and uploaded, because the answer depends on the
        // parameter values and a weight update may change it.
        std::vector<int> ipk;
        std::vector<float> spk, bpk8, wpk, bpk;
        Conv1I8Info info;
        conv1_i8_pack(w->conv_w[ti], w->conv_b[ti], C, cfg->obs_sub, cfg->obs_mul, false, ipk, spk, bpk8,
                      &info);
        conv1_mfma_pack(w->conv_w[ti], w->conv_b[ti], C, cfg->obs_sub, cfg->obs_mul, wpk, bpk);
        L.ipk = bld.upload(ipk);
        L.spk = bld.upload(spk);
        L.bpk8 = bld.upload(bpk8);
        L.wpk = bld.upload(wpk);
        L.bpk = bld.upload(bpk);
        L.planes = 3;
        const bool digits = sw.conv1 == 2 || (sw.conv1 == 0 && info.ratio3 <= 1.0);
        L.impl = digits ? CONV1_U8_I8 : CONV1_U8_MFMA;
        p->conv1_ratio2 = info.ratio2;
        p->conv1_ratio3 = info.ratio3;
      }
      if (L.impl == CONV_GENERIC) L.w_khwc_o = bld.pack_conv(w->conv_w[ti], cout, C, k);
      ++ti;
      int64_t m = (int64_t)L.Ho * L.Wo * cout * C * k * k;
      Op op{OP_CONV, name, 2 * m, (int)p->convs.size(), in_buf, out_buf, resid_buf, 0, 0, 0};
      p->convs.push_back(L);
      p->ops.push_back(op);
      macs += m;
      size_t e = (size_t)L.Ho * L.Wo * cout;
      if (e > act_elems) act_elems = e;
      C = cout; H = L.Ho; W = L.Wo;
    };
    char name[64];
    if (cfg->encoder == SF_ENCODER_CONV) {
      int in_buf = -1, out_buf = 0;
      for (int l = 0; l < cfg->n_conv; ++l) {
        snprintf(name, sizeof(name), "conv%d", l + 1);
        add_conv(name, cfg->conv[l].cout, cfg->conv[l].k, cfg->conv[l].stride, cfg->conv[l].pad,
                 0, 1, in_buf, out_buf, -1);
        in_buf = out_buf;
        out_buf ^= 1;
      }
      p->enc_buf = in_buf;
      // bf16 configuration of the benchmark shape: the first two layers as one launch (the first
      // layer's output stays in LDS); its buffer is kept for the cases that run them separately
      if (cfg->n_conv >= 2 && !sw.no_conv12_fuse && p->convs[0].impl == CONV1_U8_I8 &&
          p->convs[1].impl == CONV_IMAGE_BF16 &&
          conv12_fused_bf16_supported(cfg->obs_c, cfg->obs_h, cfg->obs_w, cfg->conv[0], cfg->conv[1])) {
        Op& a = p->ops[0];
        const Op b = p->ops[1];
        a.name = "conv1+conv2";
        a.flops_per_row += b.flops_per_row;
        a.mid_buf = a.out_buf;
        a.out_buf = b.out_buf;
        p->ops.erase(p->ops.begin() + 1);
      }
    } else {
      // buffer roles rotate: x holds the stage state, t and u are scratch
      int x = 0, t = 1, u = 2;
      int in_buf = -1;
      // With fp16 activations throughout, a stage convolution and its max-pool run as one
      // kernel, and so does each residual block.
      const bool fuse = p->bf16_path && p->act_f16 && !p->stream_f32 && !sw.no_patch_conv &&
                        !sw.no_fused_resnet;
      for (int s = 0; s < cfg->n_stage; ++s) {
        if (fuse && conv3x3_pool_supported(C, cfg->stage_ch[s], W)) {
          const int Hin = H, Win = W, C_in_stage = C;
          snprintf(name, sizeof(name), "stage%d.conv_pool", s + 1);
          // in_buf is the previous stage's x: the pooled result goes to t, which becomes x
          add_conv(name, cfg->stage_ch[s], 3, 1, 1, 0, 0, in_buf, t, -1);
          p->convs.back().impl = p->convs.back().wsp ? STEM_POOL : CONV3X3_POOL;
          if (in_buf >= 0 && !sw.no_conv_pool_regs && conv_pool_regs_supported(C_in_stage, cfg->stage_ch[s], Hin, Win))
            p->convs.back().impl = CONV_POOL_REGS;
          {
            const int tmp = x;
            x = t;
            t = tmp;
          }
          H = (Hin - 1) / 2 + 1;
          W = (Win - 1) / 2 + 1;
        } else {
          snprintf(name, sizeof(name), "stage%d.conv", s + 1);
          add_conv(name, cfg->stage_ch[s], 3, 1, 1, 0, 0, in_buf, t, -1);
          snprintf(name, sizeof(name), "stage%d.pool", s + 1);
          p->ops.push_back(Op{OP_POOL, name, 0, -1, t, x, -1, C, H, W});
          H = (H - 1) / 2 + 1;
          W = (W - 1) / 2 + 1;
        }
        const size_t first_block_op = p->ops.size();
        for (int b = 0; b < cfg->blocks_per_stage; ++b) {
          bool last = (s == cfg->n_stage - 1) && (b == cfg->blocks_per_stage - 1);
          snprintf(name, sizeof(name), "stage%d.block%d.conv_a", s + 1, b + 1);
          add_conv(name, cfg->stage_ch[s], 3, 1, 1, 1, 1, x, t, -1);
          snprintf(name, sizeof(name), "stage%d.block%d.conv_b", s + 1, b + 1);
          add_conv(name, cfg->stage_ch[s], 3, 1, 1, 0, last ? 1 : 0, t, u, x);
          if (fuse && res_block_supported(cfg->stage_ch[s])) {
            // merge the two operations: x -> u in one launch
            const Op ob = p->ops.back();
            p->ops.pop_back();
            Op& oa = p->ops.back();
            snprintf(name, sizeof(name), "stage%d.block%d", s + 1, b + 1);
            oa.name = name;
            oa.flops_per_row += ob.flops_per_row;
            oa.out_buf = u;
            p->convs[oa.conv].impl = RES_BLOCK;
          }
          int tmp = x;
          x = u;
          u = tmp;
        }
        // all blocks of the stage as one launch with the frame resident in LDS
        if (fuse && !sw.no_res_stage && cfg->blocks_per_stage >= 1 &&
            p->ops.size() - first_block_op == (size_t)cfg->blocks_per_stage &&
            res_stage_supported(cfg->stage_ch[s], H, W, cfg->blocks_per_stage)) {
          Op merged = p->ops[first_block_op];
          bool all_blocks = true;
          int64_t fl = 0;
          for (size_t i = first_block_op; i < p->ops.size(); ++i) {
            all_blocks = all_blocks && p->convs[p->ops[i].conv].impl == RES_BLOCK;
            fl += p->ops[i].flops_per_row;
          }
          if (all_blocks) {
            snprintf(name, sizeof(name), "stage%d.blocks", s + 1);
            merged.name = name;
            merged.flops_per_row = fl;
            merged.n_sub = 2 * cfg->blocks_per_stage;
            // the stage's output goes to a buffer other than its input
            if (x == merged.in_buf) {
              const int tmp = x;
              x = t;
              t = tmp;
            }
            merged.out_buf = x;
            p->convs[merged.conv].impl = RES_STAGE;
            p->ops.resize(first_block_op);
            p->ops.push_back(merged);
          }
        }
        in_buf = x;
      }
      p->enc_buf = x;
    }
  }
  p->act_elems = act_elems;
  // bytes per batch row of the largest tensor any encoder launch writes
  size_t act_row_bytes = 0;
  for (const Op& op : p->ops) {
    size_t bytes = 0;
    if (op.kind == OP_CONV) {
      const ConvLayer& L = p->convs[op.conv];
      size_t elems = (size_t)L.Ho * L.Wo * L.cout;
      if (L.impl == CONV3X3_POOL || L.impl == STEM_POOL || L.impl == CONV_POOL_REGS) elems = (size_t)((L.Ho - 1) / 2 + 1) * ((L.Wo - 1) / 2 + 1) * L.cout;
      bytes = elems * (p->bf16_path && !L.out_f32 ? 2 : 4);
    } else if (op.kind == OP_POOL) {
      bytes = (size_t)((op.H - 1) / 2 + 1) * ((op.W - 1) / 2 + 1) * op.C * (p->bf16_path && !p->stream_f32 ? 2 : 4);
    }
    if (bytes > act_row_bytes) act_row_bytes = bytes;
  }
  act_row_bytes = (act_row_bytes + 15) & ~(size_t)15;
  // Every encoder launch reads neighbouring pixels of its input from other workgroups' tiles:
  // none may write the buffer it reads.
  for (const Op& op : p->ops)
    if ((op.kind == OP_CONV || op.kind == OP_POOL) &&
        (op.out_buf == op.in_buf || (op.resid_buf >= 0 && op.out_buf == op.resid_buf))) {
      set_error("sf_policy_create: internal error: encoder launch '%s' would run in place", op.name.c_str());
      return SF_ERR_SHAPE;
    }

  // ---- FC: columns permuted from (c, y, x) to the channels-last order (y, x, c), transposed ----
  {
    // u: [fc][flat in channels-last order]
    std::vector<float> u((size_t)p->flat * cfg->fc_dim);
    for (int o = 0; o < cfg->fc_dim; ++o) {
      const float* src = w->fc_w + (size_t)o * p->flat;
      float* dst = u.data() + (size_t)o * p->flat;
      for (int c = 0; c < Cf; ++c)
        for (int yx = 0; yx < Hf * Wf; ++yx) dst[(size_t)yx * Cf + c] = bld.q(src[(size_t)c * Hf * Wf + yx]);
    }
    p->fc_b = bld.pack_vec(w->fc_b, cfg->fc_dim);
    p->fc_wt = nullptr;
    p->fc_w_t = nullptr;
    const bool fc_mfma = !sw.force_generic && !p->bf16_path &&
                         gemm_mfma_supported(p->flat, 1, 0, cfg->fc_dim);
    if (fc_mfma) {
      p->fc_wt = bld.upload(u);
      p->fc_tile = sw.fc_tile > 0 ? sw.fc_tile
                                  : gemm_mfma_pick_tile(cfg->max_batch, cfg->fc_dim, p->flat, p->flat);
    } else if (!p->bf16_path) {
      // the shape-agnostic kernel reads the transposed matrix [flat][fc]
      std::vector<float> t((size_t)p->flat * cfg->fc_dim);
      for (int o = 0; o < cfg->fc_dim; ++o)
        for (int i = 0; i < p->flat; ++i) t[(size_t)i * cfg->fc_dim + o] = u[(size_t)o * p->flat + i];
      p->fc_w_t = bld.upload(t);
    }
    p->fc_wbf = nullptr;
    if (p->bf16_path) {
      // the FC is a 1x1 "convolution" over a 1x1 image with flat channels: u is [fc][flat][1][1]
      std::vector<uint16_t> wt;
      std::vector<float> bb;
      std::vector<float> fb(cfg->fc_dim);
      for (int o = 0; o < cfg->fc_dim; ++o) fb[o] = bld.q(w->fc_b[o]);
      conv_bf16_pack(u.data(), fb.data(), cfg->fc_dim, p->flat, 1, p->act_f16, wt, bb, &p->fc_Kpad);
      p->fc_wbf = bld.upload(wt);
      p->fc_bbf = bld.upload(bb);
    }
    macs += (int64_t)p->flat * cfg->fc_dim;
    p->ops.push_back(Op{OP_FC, "fc", 2 * (int64_t)p->flat * cfg->fc_dim, -1, p->enc_buf, -1, -1, 0, 0, 0});
  }
  // ---- measurement encoder (full architecture): FC + ReLU layers, any sizes ----
  p->n_meas = cfg->meas_dim > 0 ? cfg->n_meas_layers : 0;
  p->meas_out_dim = 0;
  {
    int n_prev = cfg->meas_dim;
    int64_t m_all = 0;
    const bool fused = p->n_meas > 0 && meas_mlp_supported(cfg->meas_dim, cfg->meas_hidden[0]);
    for (int l = 0; l < p->n_meas; ++l) {
      const int n_out = cfg->meas_hidden[l];
      p->meas_w_t[l] = bld.pack_transposed(w->meas_w[l], n_out, n_prev);
      p->meas_b[l] = bld.pack_vec(w->meas_b[l], n_out);
      p->meas_in_dim[l] = n_prev;
      macs += (int64_t)n_out * n_prev;
      m_all += (int64_t)n_out * n_prev;
      if (!fused) {
        char nm[32];
        snprintf(nm, sizeof(nm), "meas.fc%d", l + 1);
        p->ops.push_back(Op{OP_MEAS, nm, 2 * (int64_t)n_out * n_prev, l, -1, -1, -1, 0, 0, 0});
      }
      n_prev = n_out;
    }
    if (fused) p->ops.push_back(Op{OP_MEAS, "meas.fc", 2 * m_all, -1, -1, -1, -1, 0, 0, 0});
    if (p->n_meas) p->meas_out_dim = n_prev;
  }
  // ---- recurrent core: its input is [FC output | encoded measurements] ----
  const bool lstm = cfg->rnn_type == SF_RNN_LSTM;
  const int core_in = cfg->fc_dim + p->meas_out_dim;
  const int HG = (lstm ? 4 : 3) * cfg->rnn_dim;
  p->state_dim = (lstm ? 2 : 1) * cfg->rnn_dim;
  p->gru_wih_t = p->gru_whh_t = nullptr;
  p->gru_wih = p->gru_whh = nullptr;
  p->rnn_seq_w = nullptr;
  p->rnn_wih_bf = p->rnn_whh_bf = nullptr;
  if (cfg->dtype == SF_DTYPE_BF16 && !sw.force_generic && !sw.no_rnn_bf16 &&
      rnn_bf16_supported(cfg->fc_dim, p->meas_out_dim, cfg->rnn_dim)) {
    // bf16 configuration: gate GEMMs on the 16-bit MFMA, state split into two bf16 terms
    std::vector<uint16_t> t;
    rnn_bf16_pack(w->rnn_w_ih, (size_t)HG * core_in, t);
    p->rnn_wih_bf = bld.upload(t);
    rnn_bf16_pack(w->rnn_w_hh, (size_t)HG * cfg->rnn_dim, t);
    p->rnn_whh_bf = bld.upload(t);
    // The FC kernel can hand its output over as bf16 (the rounding this kernel would apply
    // while staging it): half the bytes for every unit tile that re-reads the rows.  Not with a
    // second input (fp32) and not where the 16-bit activations are fp16.
    p->fc_out_bf16 = p->fc_wbf && !p->act_f16 && p->meas_out_dim == 0 && !sw.fc_out_f32;
  } else if (sw.force_generic || !rnn_mfma_supported(cfg->fc_dim, p->meas_out_dim, cfg->rnn_dim)) {
    p->gru_wih_t = bld.pack_transposed(w->rnn_w_ih, HG, core_in);
    p->gru_whh_t = bld.pack_transposed(w->rnn_w_hh, HG, cfg->rnn_dim);
  } else {
    p->gru_wih = bld.pack_vec(w->rnn_w_ih, (size_t)HG * core_in);
    p->gru_whh = bld.pack_vec(w->rnn_w_hh, (size_t)HG * cfg->rnn_dim);
    p->gru_bm = sw.gru_bm > 0 ? sw.gru_bm : rnn_mfma_pick_bm(cfg->max_batch, cfg->rnn_dim);
    p->rnn_plain_loops = sw.no_rnn_pairs ? 0 : 1;
  }
  if ((p->gru_wih || p->rnn_wih_bf) && !sw.no_rnn_seq &&
      rnn_seq_supported(cfg->fc_dim, p->meas_out_dim, cfg->rnn_dim)) {
    // the same matrices once more (fp32 values; in a bf16 configuration the rounded ones), in the
    // operand order of the kernel that runs the core on the few rows per time step of
    // sf_policy_unroll
    std::vector<float> qi((size_t)HG * core_in), qh((size_t)HG * cfg->rnn_dim), t;
    for (size_t i = 0; i < qi.size(); ++i) qi[i] = bld.q(w->rnn_w_ih[i]);
    for (size_t i = 0; i < qh.size(); ++i) qh[i] = bld.q(w->rnn_w_hh[i]);
    rnn_seq_pack(qi.data(), qh.data(), core_in, cfg->rnn_dim, lstm ? 1 : 0, t);
    p->rnn_seq_w = bld.upload(t);
  }
  p->gru_bih = bld.pack_vec(w->rnn_b_ih, HG);
  p->gru_bhh = bld.pack_vec(w->rnn_b_hh, HG);
  macs += (int64_t)HG * (core_in + cfg->rnn_dim);
  p->ops.push_back(Op{OP_GRU, lstm ? "lstm" : "gru", 2 * (int64_t)HG * (core_in + cfg->rnn_dim), -1, -1, -1,
                      -1, 0, 0, 0});
  // ---- heads: action logits then the value row ----
  {
    int sumA = 0;
    std::vector<int32_t> off(cfg->n_heads + 1, 0);
    for (int k = 0; k < cfg->n_heads; ++k) {
      sumA += cfg->head_sizes[k];
      off[k + 1] = sumA;
    }
    p->sumA = sumA;
    p->max_head = 0;
    for (int k = 0; k < cfg->n_heads; ++k)
      if (cfg->head_sizes[k] > p->max_head) p->max_head = cfg->head_sizes[k];
    const int Hd = cfg->rnn_dim;
    std::vector<float> hw((size_t)(sumA + 1) * Hd), hb(sumA + 1);
    for (size_t i = 0; i < (size_t)sumA * Hd; ++i) hw[i] = bld.q(w->pi_w[i]);
    for (int i = 0; i < Hd; ++i) hw[(size_t)sumA * Hd + i] = bld.q(w->v_w[i]);
    for (int i = 0; i < sumA; ++i) hb[i] = bld.q(w->pi_b[i]);
    hb[sumA] = bld.q(w->v_b[0]);
    p->head_w = bld.upload(hw);
    p->head_b = bld.upload(hb);
    p->head_off = bld.upload(off);
    macs += (int64_t)(sumA + 1) * Hd;
    p->ops.push_back(Op{OP_HEADS, "heads", 2 * (int64_t)(sumA + 1) * Hd, -1, -1, -1, -1, 0, 0, 0});
  }
  p->flops_per_row = 2 * macs;

  // ---- workspace ----
  int n_act = cfg->encoder == SF_ENCODER_RESNET ? 3 : 2;
  for (int i = 0; i < 3; ++i)
    p->act[i] = i < n_act ? (float*)bld.dev_alloc(act_row_bytes * cfg->max_batch)
                          : nullptr;
  p->trash = (float*)bld.dev_alloc(256);
  p->fc_out = (float*)bld.dev_alloc(sizeof(float) * (size_t)cfg->fc_dim * cfg->max_batch);
  p->h_new = (float*)bld.dev_alloc(sizeof(float) * (size_t)p->state_dim * cfg->max_batch);
  for (int l = 0; l < p->n_meas; ++l)
    p->meas_buf[l] = (float*)bld.dev_alloc(sizeof(float) * (size_t)cfg->meas_hidden[l] * cfg->max_batch);

  return bld.status;
}

// First non-finite value of a tensor, or -1.
long long first_non_finite(const float* v, size_t n) {
  for (size_t i = 0; i < n; ++i) {
    uint32_t u;
    memcpy(&u, &v[i], 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return (long long)i;
  }
  return -1;
}

// Every parameter must be a finite number; in the residual encoder of a bf16 configuration
// (16-bit operands in fp16) the encoder and FC weights must also fit fp16's range.
int check_values(const sf_policy_config* cfg, const sf_policy_weights* w, int flat, const char* fn) {
  struct Tensor {
    const char* name;
    int index;
    const float* v;
    size_t n;
    bool fp16_operand;
  };
  std::vector<Tensor> ts;
  const bool f16 = cfg->dtype == SF_DTYPE_BF16 && cfg->encoder == SF_ENCODER_RESNET;
  int C = cfg->obs_c, ti = 0;
  if (cfg->encoder == SF_ENCODER_CONV) {
    for (int l = 0; l < cfg->n_conv; ++l, ++ti) {
      const sf_conv& v = cfg->conv[l];
      ts.push_back({"conv_w", ti, w->conv_w[ti], (size_t)v.cout * C * v.k * v.k, false});
      ts.push_back({"conv_b", ti, w->conv_b[ti], (size_t)v.cout, false});
      C = v.cout;
    }
  } else {
    for (int st = 0; st < cfg->n_stage; ++st) {
      for (int j = 0; j < 1 + 2 * cfg->blocks_per_stage; ++j, ++ti) {
        const int cin = j == 0 ? C : cfg->stage_ch[st];
        ts.push_back({"conv_w", ti, w->conv_w[ti], (size_t)cfg->stage_ch[st] * cin * 9, f16});
        ts.push_back({"conv_b", ti, w->conv_b[ti], (size_t)cfg->stage_ch[st], false});
      }
      C = cfg->stage_ch[st];
    }
  }
  const int G = cfg->rnn_type == SF_RNN_LSTM ? 4 : 3;
  int core_in = cfg->fc_dim, n_prev = cfg->meas_dim;
  for (int l = 0; cfg->meas_dim > 0 && l < cfg->n_meas_layers; ++l) {
    ts.push_back({"meas_w", l, w->meas_w[l], (size_t)cfg->meas_hidden[l] * n_prev, false});
    ts.push_back({"meas_b", l, w->meas_b[l], (size_t)cfg->meas_hidden[l], false});
    n_prev = cfg->meas_hidden[l];
  }
  if (cfg->meas_dim > 0) core_in += n_prev;
  int sumA = 0;
  for (int k = 0; k < cfg->n_heads; ++k) sumA += cfg->head_sizes[k];
  const size_t H = (size_t)cfg->rnn_dim;
  ts.push_back({"fc_w", 0, w->fc_w, (size_t)cfg->fc_dim * flat, f16});
  ts.push_back({"fc_b", 0, w->fc_b, (size_t)cfg->fc_dim, false});
  ts.push_back({"rnn_w_ih", 0, w->rnn_w_ih, G * H * core_in, false});
  ts.push_back({"rnn_w_hh", 0, w->rnn_w_hh, G * H * H, false});
  ts.push_back({"rnn_b_ih", 0, w->rnn_b_ih, G * H, false});
  ts.push_back({"rnn_b_hh", 0, w->rnn_b_hh, G * H, false});
  ts.push_back({"pi_w", 0, w->pi_w, (size_t)sumA * H, false});
  ts.push_back({"pi_b", 0, w->pi_b, (size_t)sumA, false});
  ts.push_back({"v_w", 0, w->v_w, H, false});
  ts.push_back({"v_b", 0, w->v_b, 1, false});
  for (const Tensor& t : ts) {
    const long long bad = first_non_finite(t.v, t.n);
    if (bad >= 0) {
      set_error("%s: %s[%d] element %lld is not finite", fn, t.name, t.index, bad);
      return SF_ERR_ARG;
    }
    if (t.fp16_operand)
      for (size_t i = 0; i < t.n; ++i)
        if (fabsf(t.v[i]) > 65280.0f) {  // the largest bf16 value that fp16 can hold
          set_error("%s: %s[%d] element %zu = %g is outside the fp16 range of the residual "
                    "encoder's 16-bit operands", fn, t.name, t.index, i, (double)t.v[i]);
          return SF_ERR_ARG;
        }
  }
  return SF_OK;
}

int check_weights(const sf_policy_config* cfg, const sf_policy_weights* w, const char* fn) {
  int n_tensors = cfg->encoder == SF_ENCODER_CONV ? cfg->n_conv
                                                  : cfg->n_stage * (1 + 2 * cfg->blocks_per_stage);
  for (int i = 0; i < n_tensors; ++i)
    if (!w->conv_w[i] || !w->conv_b[i]) {
      set_error("%s: conv tensor %d is null", fn, i);
      return SF_ERR_ARG;
    }
  if (!w->fc_w || !w->fc_b || !w->rnn_w_ih || !w->rnn_w_hh || !w->rnn_b_ih || !w->rnn_b_hh ||
      !w->pi_w || !w->pi_b || !w->v_w || !w->v_b) {
    set_error("%s: a weight pointer is null", fn);
    return SF_ERR_ARG;
  }
  for (int l = 0; cfg->meas_dim > 0 && l < cfg->n_meas_layers; ++l)
    if (!w->meas_w[l] || !w->meas_b[l]) {
      set_error("%s: measurement layer %d has a null weight pointer", fn, l);
      return SF_ERR_ARG;
    }
  return SF_OK;
}

}  // namespace

extern "C" const char* sf_last_error(void) { return g_err; }

extern "C" int sf_policy_create(const sf_policy_config* cfg, const sf_policy_weights* w,
                                int hip_device, sf_policy** out) {
  if (out) *out = nullptr;
  if (!cfg || !w || !out) {
    set_error("sf_policy_create: null argument");
    return SF_ERR_ARG;
  }
  if (cfg->struct_size != sizeof(sf_policy_config) || cfg->abi_version != SF_ABI_VERSION) {
    set_error("sf_policy_create: struct_size %u / abi_version %u do not match this library (%zu / %u)",
              cfg->struct_size, cfg->abi_version, sizeof(sf_policy_config), SF_ABI_VERSION);
    return SF_ERR_ARG;
  }
  int Cf, Hf, Wf;
  int rc = check_config(cfg, &Cf, &Hf, &Wf);
  if (rc != SF_OK) return rc;

  // every parameter tensor the description needs must be present
  rc = check_weights(cfg, w, "sf_policy_create");
  if (rc != SF_OK) return rc;
  rc = check_values(cfg, w, Cf * Hf * Wf, "sf_policy_create");
  if (rc != SF_OK) return rc;

  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || hip_device < 0 || hip_device >= n_dev) {
    set_error("sf_policy_create: HIP device %d not available (%d devices)", hip_device, n_dev);
    return SF_ERR_DEVICE;
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, hip_device) != hipSuccess) {
    set_error("sf_policy_create: hipGetDeviceProperties failed");
    return SF_ERR_DEVICE;
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
    set_error("sf_policy_create: device %d is %s; this library is built for gfx950 only",
              hip_device, prop.gcnArchName);
    return SF_ERR_ARCH;
  }
  if (hipSetDevice(hip_device) != hipSuccess) {
    set_error("sf_policy_create: hipSetDevice(%d) failed", hip_device);
    return SF_ERR_DEVICE;
  }

  Policy* p = new (std::nothrow) Policy();
  if (!p) {
    set_error("sf_policy_create: out of host memory");
    return SF_ERR_OOM;
  }
  p->device = hip_device;
  p->sw = read_switches();
  Builder bld{p, cfg->dtype == SF_DTYPE_BF16};
  bld.status = build_policy(p, cfg, w, bld, Cf, Hf, Wf);
  p->events.resize(p->ops.size() + 1, nullptr);
  for (auto& ev : p->events)
    if (bld.status == SF_OK && hipEventCreate(&ev) != hipSuccess) {
      set_error("sf_policy_create: hipEventCreate failed");
      bld.status = SF_ERR_DEVICE;
    }
  if (bld.status != SF_OK) {
    int st = bld.status;
    free_policy(p);
    return st;
  }
  if (hipDeviceSynchronize() != hipSuccess) {
    set_error("sf_policy_create: device synchronisation failed");
    free_policy(p);
    return SF_ERR_DEVICE;
  }
  *out = reinterpret_cast<sf_policy*>(p);
  return SF_OK;
}

extern "C" int sf_policy_update_weights(sf_policy* handle, const sf_policy_weights* w, void* hip_stream) {
  static const char* fn = "sf_policy_update_weights";
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p || !w) {
    set_error("%s: null argument", fn);
    return SF_ERR_ARG;
  }
  int rc = check_weights(&p->cfg, w, fn);
  if (rc != SF_OK) return rc;
  rc = check_values(&p->cfg, w, p->flat, fn);
  if (rc != SF_OK) return rc;
  if (hipSetDevice(p->device) != hipSuccess) {
    set_error("%s: hipSetDevice(%d) failed", fn, p->device);
    return SF_ERR_DEVICE;
  }
  if (!p->stage) {
    // the event first: the staging area is published only together with its event
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      set_error("%s: hipEventCreate failed", fn);
      return SF_ERR_DEVICE;
    }
    unsigned char* stage = nullptr;
    if (hipHostMalloc((void**)&stage, p->upload_bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipEventDestroy(ev);
      set_error("%s: page-locked staging allocation of %zu bytes failed", fn, p->upload_bytes);
      return SF_ERR_OOM;
    }
    p->stage_ev = ev;
    p->stage = stage;
    p->stage_bytes = p->upload_bytes;
  } else if (hipEventSynchronize(p->stage_ev) != hipSuccess) {  // the previous update's copies
    set_error("%s: waiting for the previous update failed", fn);
    return SF_ERR_DEVICE;
  }
  int Cf, Hf, Wf;
  rc = check_config(&p->cfg, &Cf, &Hf, &Wf);
  if (rc != SF_OK) return rc;
  // Pack the whole plan into the staging area and check it against the live policy before
  // any copy is enqueued: a failure up to here leaves the live parameters untouched.
  Policy scratch{};  // receives a copy of the plan; owns nothing (value-initialised: zeros)
  scratch.device = p->device;
  scratch.sw = p->sw;  // the switches as they were at create, whatever the environment says now
  Builder bld{&scratch, p->cfg.dtype == SF_DTYPE_BF16};
  bld.target = p;
  rc = build_policy(&scratch, &p->cfg, w, bld, Cf, Hf, Wf);
  if (rc != SF_OK) return rc;
  if (bld.next != p->allocations.size()) {
    set_error("%s: the update visited %zu of the policy's %zu buffers", fn, bld.next, p->allocations.size());
    return SF_ERR_SHAPE;
  }
  bool same_plan = scratch.convs.size() == p->convs.size() && scratch.ops.size() == p->ops.size() &&
                   scratch.bf16_path == p->bf16_path && scratch.act_f16 == p->act_f16 &&
                   scratch.stream_f32 == p->stream_f32 && scratch.fc_tile == p->fc_tile &&
                   scratch.fc_out_bf16 == p->fc_out_bf16 && (scratch.fc_wt != nullptr) == (p->fc_wt != nullptr) &&
                   (scratch.fc_wbf != nullptr) == (p->fc_wbf != nullptr) &&
                   (scratch.gru_wih != nullptr) == (p->gru_wih != nullptr) &&
                   scratch.rnn_seq_w == p->rnn_seq_w &&
                   (scratch.rnn_wih_bf != nullptr) == (p->rnn_wih_bf != nullptr);
  for (size_t i = 0; same_plan && i < p->convs.size(); ++i) {
    const ConvLayer &a = scratch.convs[i], &b = p->convs[i];
    // the first convolution's arithmetic (digit planes or fp32) follows the parameter values
    const bool conv1_pair = (a.impl == CONV1_U8_I8 || a.impl == CONV1_U8_MFMA) &&
                            (b.impl == CONV1_U8_I8 || b.impl == CONV1_U8_MFMA) && a.ipk && a.wpk;
    same_plan = (a.impl == b.impl || conv1_pair) && a.tile == b.tile && a.wpk == b.wpk && a.wbf == b.wbf &&
                a.ipk == b.ipk && a.w_khwc_o == b.w_khwc_o && a.wsp == b.wsp;
  }
  if (!same_plan) {
    set_error("%s: internal error: the replayed plan differs from the one built at create", fn);
    return SF_ERR_SHAPE;
  }
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  rc = bld.flush(stream);
  if (rc == SF_OK)
    for (size_t i = 0; i < p->convs.size(); ++i) {
      p->convs[i].impl = scratch.convs[i].impl;
      p->convs[i].planes = scratch.convs[i].planes;
    }
  p->conv1_ratio2 = scratch.conv1_ratio2;
  p->conv1_ratio3 = scratch.conv1_ratio3;
  // recorded also after a failed copy, so that the next update waits for whatever was enqueued
  if (hipEventRecord(p->stage_ev, stream) != hipSuccess && rc == SF_OK) {
    set_error("%s: hipEventRecord failed", fn);
    rc = SF_ERR_DEVICE;
  }
  return rc;
}

extern "C" int sf_policy_destroy(sf_policy* handle) {
  free_policy(reinterpret_cast<Policy*>(handle));
  return SF_OK;
}

extern "C" int64_t sf_policy_flops_per_row(const sf_policy* handle) {
  return handle ? reinterpret_cast<const Policy*>(handle)->flops_per_row : 0;
}

#define SF_LAUNCH(expr)                                                         \
  do {                                                                          \
    hipError_t e_ = (expr);                                                     \
    if (e_ != hipSuccess) {                                                     \
      set_error("sf_policy_step: %s failed: %s", #expr, hipGetErrorString(e_)); \
      return SF_ERR_DEVICE;                                                     \
    }                                                                           \
  } while (0)

namespace {

// The launch sequence of one step.  h_in / h_out are row-indexed by the batch row, unless
// ids is given: then row b reads its state from h_in[ids[b]] (a table of n_env rows), and
// the heads launch copies the new state from h_out[b] to h_table[ids[b]].
// `parts` selects which launches run: the encoder (everything before the core), the core, the
// heads.  The core reads its input rows starting at row `feat_row` of the encoder's output.
enum : unsigned { PART_ENCODER = 1u, PART_CORE = 2u, PART_HEADS = 4u, PART_ALL = 7u };
int run_step(Policy* p, int32_t B, const uint8_t* obs, const float* meas, const float* h_in,
             const uint8_t* done, uint64_t seed, uint64_t step, int32_t* actions, float* logp,
             float* value, float* h_out, float* logits_opt, const int32_t* ids, float* h_table,
             int n_env, hipStream_t st, unsigned parts = PART_ALL, size_t feat_row = 0);

bool misaligned(const void* q, uintptr_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) != 0; }

}  // namespace

extern "C" int sf_policy_step(sf_policy* handle, int32_t B, const uint8_t* obs, const float* meas,
                              const float* h_in, const uint8_t* done, uint64_t seed, uint64_t step,
                              int32_t* actions, float* logp, float* value, float* h_out,
                              float* logits_opt, void* hip_stream) {
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p) {
    set_error("sf_policy_step: null handle");
    return SF_ERR_ARG;
  }
  const sf_policy_config& c = p->cfg;
  if (B < 0 || B > c.max_batch) {
    set_error("sf_policy_step: B = %d outside [0, max_batch = %d]", B, c.max_batch);
    return SF_ERR_BATCH;
  }
  if (B == 0) return SF_OK;
  if (!obs || !h_in || !done || !actions || !logp || !value || !h_out || (c.meas_dim > 0 && !meas)) {
    set_error("sf_policy_step: null buffer");
    return SF_ERR_ARG;
  }
  if (misaligned(obs, 4) || (c.meas_dim > 0 && misaligned(meas, 4)) || misaligned(h_in, 16) || misaligned(h_out, 16) || misaligned(actions, 4) ||
      misaligned(logp, 4) || misaligned(value, 4) || (logits_opt && misaligned(logits_opt, 4))) {
    set_error("sf_policy_step: misaligned buffer (obs, actions, logp, value, logits: 4 bytes; "
              "h_in, h_out: 16 bytes)");
    return SF_ERR_ARG;
  }
  {
    uintptr_t a0 = (uintptr_t)h_in, b0 = (uintptr_t)h_out;
    uintptr_t n = sizeof(float) * (uintptr_t)B * p->state_dim;
    if (a0 < b0 + n && b0 < a0 + n) {
      set_error("sf_policy_step: h_out overlaps h_in");
      return SF_ERR_ALIAS;
    }
  }
  return run_step(p, B, obs, meas, h_in, done, seed, step, actions, logp, value, h_out, logits_opt,
                  nullptr, nullptr, 0, reinterpret_cast<hipStream_t>(hip_stream));
}

extern "C" int sf_policy_step_indexed(sf_policy* handle, int32_t B, const uint8_t* obs,
                                      const float* meas, float* h_table, int32_t n_env,
                                      const int32_t* env_ids, const uint8_t* done,
                                      uint64_t seed, uint64_t step, int32_t* actions, float* logp,
                                      float* value, float* logits_opt, void* hip_stream) {
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p) {
    set_error("sf_policy_step_indexed: null handle");
    return SF_ERR_ARG;
  }
  const sf_policy_config& c = p->cfg;
  if (B < 0 || B > c.max_batch) {
    set_error("sf_policy_step_indexed: B = %d outside [0, max_batch = %d]", B, c.max_batch);
    return SF_ERR_BATCH;
  }
  if (n_env < 1) {
    set_error("sf_policy_step_indexed: n_env = %d, must be at least 1", n_env);
    return SF_ERR_ARG;
  }
  if (B == 0) return SF_OK;
  if (!obs || !h_table || !env_ids || !done || !actions || !logp || !value || (c.meas_dim > 0 && !meas)) {
    set_error("sf_policy_step_indexed: null buffer");
    return SF_ERR_ARG;
  }
  if (misaligned(obs, 4) || (c.meas_dim > 0 && misaligned(meas, 4)) || misaligned(h_table, 16) || misaligned(env_ids, 4) || misaligned(actions, 4) ||
      misaligned(logp, 4) || misaligned(value, 4) || (logits_opt && misaligned(logits_opt, 4))) {
    set_error("sf_policy_step_indexed: misaligned buffer (obs, env_ids, actions, logp, value, logits: "
              "4 bytes; h_table: 16 bytes)");
    return SF_ERR_ARG;
  }
  return run_step(p, B, obs, meas, h_table, done, seed, step, actions, logp, value, p->h_new, logits_opt,
                  env_ids, h_table, n_env, reinterpret_cast<hipStream_t>(hip_stream));
}

namespace {

int run_step(Policy* p, int32_t B, const uint8_t* obs, const float* meas, const float* h_in,
             const uint8_t* done, uint64_t seed, uint64_t step, int32_t* actions, float* logp,
             float* value, float* h_out, float* logits_opt, const int32_t* ids, float* h_table,
             int n_env, hipStream_t st, unsigned parts, size_t feat_row) {
  const sf_policy_config& c = p->cfg;
  auto buf = [&](int i) -> float* { return i < 0 ? nullptr : p->act[i]; };
  const bool timing = p->timing && parts == PART_ALL;
  if (timing) SF_LAUNCH(hipEventRecord(p->events[0], st));
  for (size_t i = 0; i < p->ops.size(); ++i) {
    const Op& op = p->ops[i];
    const unsigned part = op.kind == OP_GRU ? PART_CORE : op.kind == OP_HEADS ? PART_HEADS : PART_ENCODER;
    if (!(parts & part)) continue;
    switch (op.kind) {
      case OP_CONV: {
        const ConvLayer& L = p->convs[op.conv];
        const void* in = op.in_buf < 0 ? (const void*)obs : (const void*)buf(op.in_buf);
        switch (L.impl) {
          case CONV1_U8_I8:
            if (op.mid_buf >= 0) {
              // first and second layer: one launch where the fused kernel applies (two digit
              // planes, 16-byte aligned frames), else the two kernels in sequence (same bits)
              const ConvLayer& L2 = p->convs[op.conv + 1];
              if (L.planes == 2 && !misaligned(obs, 16)) {
                SF_LAUNCH(launch_conv12_fused_bf16(L, L2, B, obs, buf(op.out_buf), st));
              } else {
                SF_LAUNCH(launch_conv1_i8(L, B, obs, L.ipk, L.spk, L.bpk8, buf(op.mid_buf), 1, L.planes,
                                          p->conv1_waves, p->conv1_image, st));
                SF_LAUNCH(launch_conv_image_bf16(buf(op.mid_buf), L2.wbf, L2.bbf, buf(op.out_buf), B, L2.H,
                                                 L2.W, L2.cin, L2.k, L2.s, L2.Ho, L2.Wo, L2.cout,
                                                 L2.relu_out, st));
              }
              break;
            }
            SF_LAUNCH(launch_conv1_i8(L, B, obs, L.ipk, L.spk, L.bpk8, buf(op.out_buf), p->bf16_path,
                                      L.planes, p->conv1_waves, p->conv1_image, st));
            break;
          case CONV1_U8_MFMA:
            SF_LAUNCH(launch_conv1_mfma(L, B, obs, L.wpk, L.bpk, buf(op.out_buf), p->trash,
                                        p->conv1_waves, c.obs_sub, st));
            break;
          case CONV_GEMM_MFMA:
            SF_LAUNCH(launch_gemm_mfma((const float*)in, L.wpk, L.bpk, buf(op.out_buf), B, L.H, L.W,
                                       L.cin, L.k, L.s, L.Ho, L.Wo, L.cout, L.relu_out, L.tile,
                                       op.conv + 1, st));
            break;
          case CONV_IMAGE_BF16:
            SF_LAUNCH(launch_conv_image_bf16(in, L.wbf, L.bbf, buf(op.out_buf), B, L.H, L.W, L.cin,
                                             L.k, L.s, L.Ho, L.Wo, L.cout, L.relu_out, st));
            break;
          case CONV_BF16:
            SF_LAUNCH(launch_conv_bf16(in, L.wbf, L.bbf, buf(op.resid_buf), buf(op.out_buf), B, L.H,
                                       L.W, L.cin, L.k, L.s, L.pad, L.Ho, L.Wo, L.cout, L.Kpad,
                                       L.relu_in, L.relu_out, L.in_f32, p->stream_f32, L.out_f32,
                                       p->act_f16, p->conv_bf16_tc, op.conv + 1, st));
            break;
          case CONV3X3_PATCH:
            SF_LAUNCH(launch_conv3x3_patch(in, L.wbf, L.bbf, buf(op.resid_buf), p->stream_f32,
                                           buf(op.out_buf), B, L.H, L.W, L.cin, L.cout, L.in_f32, L.relu_in, L.relu_out,
                                           L.out_f32, p->act_f16, st));
            break;
          case CONV3X3_POOL:
            SF_LAUNCH(launch_conv3x3_pool(in, L.wbf, L.bbf, buf(op.out_buf), B, L.H, L.W, L.cin, L.cout,
                                          c.obs_sub, c.obs_mul, st));
            break;
          case CONV_POOL_REGS:
            SF_LAUNCH(launch_conv_pool_regs(in, L.wbf, L.bbf, buf(op.out_buf), B, L.H, L.W, L.cin, st));
            break;
          case STEM_POOL:
            SF_LAUNCH(launch_stem_pool(obs, L.wsp, L.bbf, buf(op.out_buf), B, L.H, L.W, c.obs_sub, c.obs_mul, st));
            break;
          case RES_STAGE: {
            const uint16_t* wpk[SF_MAX_CONV_TENSORS];
            const float* bias[SF_MAX_CONV_TENSORS];
            for (int k = 0; k < op.n_sub; ++k) {
              wpk[k] = L.cin == 16 ? p->convs[op.conv + k].wsp : p->convs[op.conv + k].wbf;
              bias[k] = p->convs[op.conv + k].bbf;
            }
            SF_LAUNCH(launch_res_stage(in, buf(op.out_buf), wpk, bias, op.n_sub, B, L.H, L.W, L.cin,
                                       p->convs[op.conv + op.n_sub - 1].relu_out, st));
            break;
          }
          case RES_BLOCK: {
            const ConvLayer& Lb = p->convs[op.conv + 1];
            SF_LAUNCH(launch_res_block(in, L.wbf, L.bbf, Lb.wbf, Lb.bbf, buf(op.out_buf), B, L.H, L.W,
                                       L.cin, Lb.relu_out, st));
            break;
          }
          case CONV3X3_STEM:
            SF_LAUNCH(launch_conv3x3_stem(obs, L.wbf, L.bbf, buf(op.out_buf), B, L.H, L.W, L.cout,
                                          c.obs_sub, c.obs_mul, p->act_f16, st));
            break;
          case CONV3X3_U8_BF16:
            SF_LAUNCH(launch_conv3x3_u8_bf16(B, L.cin, L.H, L.W, L.cout, obs, L.w_cpqo, L.bias,
                                             buf(op.out_buf), c.obs_sub, c.obs_mul, p->act_f16, st));
            break;
          default:
            SF_LAUNCH(launch_conv_generic(L, B, in, op.in_buf < 0, c.obs_sub, c.obs_mul,
                                          buf(op.resid_buf), buf(op.out_buf), st));
        }
        break;
      }
      case OP_POOL:
        if (p->bf16_path)
          SF_LAUNCH(launch_maxpool_bf16(B, op.C, op.H, op.W, buf(op.in_buf), buf(op.out_buf),
                                        p->stream_f32, p->act_f16, st));
        else
          SF_LAUNCH(launch_maxpool3x3s2p1(B, op.C, op.H, op.W, buf(op.in_buf), buf(op.out_buf), st));
        break;
      case OP_FC:
        if (p->fc_wbf)
          SF_LAUNCH(launch_conv_bf16(buf(op.in_buf), p->fc_wbf, p->fc_bbf, nullptr, p->fc_out, B, 1, 1,
                                     p->flat, 1, 1, 0, 1, 1, c.fc_dim, p->fc_Kpad, 0, 1,
                                     p->stream_f32, 0, p->fc_out_bf16 ? 0 : 1, p->act_f16,
                                     p->conv_bf16_tc, 0, st));
        else if (p->fc_wt)
          SF_LAUNCH(launch_gemm_mfma(buf(op.in_buf), p->fc_wt, p->fc_b, p->fc_out, B, 1, 1, p->flat, 1,
                                     1, 1, 1, c.fc_dim, 1, p->fc_tile, 0, st));
        else
          SF_LAUNCH(launch_linear_generic(B, p->flat, c.fc_dim, buf(op.in_buf), p->fc_w_t, p->fc_b,
                                          1, p->fc_out, st));
        break;
      case OP_MEAS: {
        const int l = op.conv;
        if (l < 0) {  // every layer in one launch
          const bool two = p->n_meas == 2;
          SF_LAUNCH(launch_meas_mlp(B, c.meas_dim, meas, p->meas_w_t[0], p->meas_b[0], c.meas_hidden[0],
                                    two ? p->meas_w_t[1] : nullptr, two ? p->meas_b[1] : nullptr,
                                    two ? c.meas_hidden[1] : 0, p->meas_buf[p->n_meas - 1], st));
          break;
        }
        SF_LAUNCH(launch_linear_generic(B, p->meas_in_dim[l], c.meas_hidden[l],
                                        l == 0 ? meas : p->meas_buf[l - 1], p->meas_w_t[l],
                                        p->meas_b[l], 1, p->meas_buf[l], st));
        break;
      }
      case OP_GRU: {
        const float* x2 = p->n_meas ? p->meas_buf[p->n_meas - 1] + feat_row * p->meas_out_dim : nullptr;
        const float* x1 = (const float*)((const char*)p->fc_out +
                                         feat_row * c.fc_dim * (p->fc_out_bf16 ? 2 : 4));
        const int lstm = c.rnn_type == SF_RNN_LSTM;
        if (parts == PART_CORE && p->rnn_seq_w && !ids)
          // (one time step of the pass over trajectories: few rows)
          SF_LAUNCH(launch_rnn_seq(lstm, B, c.fc_dim, p->meas_out_dim, c.rnn_dim, x1, p->fc_out_bf16, x2, h_in, done,
                                   p->rnn_seq_w, p->gru_bih, p->gru_bhh, h_out, st));
        else if (p->rnn_wih_bf)
          SF_LAUNCH(launch_rnn_bf16(lstm, B, c.fc_dim, p->meas_out_dim, c.rnn_dim, x1,
                                    p->fc_out_bf16, x2, h_in, done, p->rnn_wih_bf, p->rnn_whh_bf, p->gru_bih, p->gru_bhh, h_out,
                                    ids, n_env, st));
        else if (p->gru_wih)
          SF_LAUNCH(launch_rnn_mfma(lstm, B, c.fc_dim, p->meas_out_dim, c.rnn_dim, x1, x2, h_in,
                                    done, p->gru_wih, p->gru_whh, p->gru_bih, p->gru_bhh, h_out,
                                    p->gru_bm, p->rnn_plain_loops, ids, n_env, st));
        else
          SF_LAUNCH(launch_rnn_generic(lstm, B, c.fc_dim, p->meas_out_dim, c.rnn_dim, x1, x2,
                                       h_in, done, p->gru_wih_t, p->gru_whh_t, p->gru_bih, p->gru_bhh,
                                       h_out, ids, n_env, st));
        break;
      }
      case OP_HEADS:
        SF_LAUNCH(launch_heads(B, c.rnn_dim, c.n_heads, p->sumA, p->head_off, h_out, p->head_w,
                               p->head_b, seed, step, actions, logp, value, logits_opt, ids, h_table,
                               n_env, p->state_dim, p->max_head, st));
        break;
    }
    if (timing) SF_LAUNCH(hipEventRecord(p->events[i + 1], st));
  }
  return SF_OK;
}

}  // namespace

extern "C" int sf_policy_unroll(sf_policy* handle, int32_t T, int32_t N, const uint8_t* obs,
                                const float* meas, const float* h0, const uint8_t* done,
                                float* logits, float* value, float* h_seq, void* hip_stream) {
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p) {
    set_error("sf_policy_unroll: null handle");
    return SF_ERR_ARG;
  }
  const sf_policy_config& c = p->cfg;
  if (T < 1 || N < 0 || (int64_t)T * N > c.max_batch) {
    set_error("sf_policy_unroll: T = %d, N = %d: need T >= 1, N >= 0 and T * N <= max_batch = %d", T, N,
              c.max_batch);
    return SF_ERR_BATCH;
  }
  if (N == 0) return SF_OK;
  if (!obs || !h0 || !done || !logits || !value || !h_seq || (c.meas_dim > 0 && !meas)) {
    set_error("sf_policy_unroll: null buffer");
    return SF_ERR_ARG;
  }
  if (misaligned(obs, 4) || (c.meas_dim > 0 && misaligned(meas, 4)) || misaligned(h0, 16) ||
      misaligned(h_seq, 16) || misaligned(logits, 4) || misaligned(value, 4)) {
    set_error("sf_policy_unroll: misaligned buffer (obs, meas, logits, value: 4 bytes; h0, h_seq: 16 bytes)");
    return SF_ERR_ARG;
  }
  // every time step's rows must start where the kernels may use 16-byte accesses
  const size_t feat_bytes = (size_t)N * c.fc_dim * (p->fc_out_bf16 ? 2 : 4);
  if (feat_bytes % 16 || ((size_t)N * p->meas_out_dim * 4) % 16 || ((size_t)N * p->state_dim * 4) % 16) {
    set_error("sf_policy_unroll: N = %d rows of features (%d), measurement features (%d) or state (%d "
              "floats) are not a multiple of 16 bytes", N, c.fc_dim, p->meas_out_dim, p->state_dim);
    return SF_ERR_SHAPE;
  }
  {
    const uintptr_t a0 = (uintptr_t)h0, b0 = (uintptr_t)h_seq;
    if (a0 < b0 + sizeof(float) * (uintptr_t)T * N * p->state_dim && b0 < a0 + sizeof(float) * (uintptr_t)N * p->state_dim) {
      set_error("sf_policy_unroll: h_seq overlaps h0");
      return SF_ERR_ALIAS;
    }
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int32_t rows = T * N;
  // the encoder on all T * N frames at once (their features stay in the handle's workspace) ...
  int rc = run_step(p, rows, obs, meas, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr,
                    nullptr, nullptr, 0, st, PART_ENCODER);
  // ... the core one time step after the other, each reading the state rows the previous wrote ...
  for (int32_t t = 0; t < T && rc == SF_OK; ++t) {
    const size_t r = (size_t)t * N;
    const float* h_prev = t == 0 ? h0 : h_seq + (r - N) * p->state_dim;
    rc = run_step(p, N, nullptr, nullptr, h_prev, done + r, 0, 0, nullptr, nullptr, nullptr,
                  h_seq + r * p->state_dim, nullptr, nullptr, nullptr, 0, st, PART_CORE, r);
  }
  // ... and the heads on all T * N states at once (no action is drawn)
  if (rc == SF_OK)
    rc = run_step(p, rows, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, value, h_seq, logits,
                  nullptr, nullptr, 0, st, PART_HEADS);
  return rc;
}

extern "C" int32_t sf_policy_state_dim(const sf_policy* handle) {
  return handle ? reinterpret_cast<const Policy*>(handle)->state_dim : 0;
}

// ---- measurement aids ------------------------------------------------------

extern "C" int sf_policy_op_count(const sf_policy* handle) {
  return handle ? (int)reinterpret_cast<const Policy*>(handle)->ops.size() : 0;
}

extern "C" const char* sf_policy_op_name(const sf_policy* handle, int i) {
  const Policy* p = reinterpret_cast<const Policy*>(handle);
  if (!p || i < 0 || i >= (int)p->ops.size()) return "";
  return p->ops[i].name.c_str();
}

extern "C" const char* sf_policy_op_kernel(const sf_policy* handle, int i) {
  const Policy* p = reinterpret_cast<const Policy*>(handle);
  if (!p || i < 0 || i >= (int)p->ops.size()) return "";
  const Op& op = p->ops[i];
  switch (op.kind) {
    case OP_CONV:
      if (op.mid_buf >= 0) return "conv12_fused";
      switch (p->convs[op.conv].impl) {
        case CONV1_U8_MFMA: return "conv1_mfma";
        case CONV_GEMM_MFMA: return "gemm_mfma";
        case CONV1_U8_I8: return "conv1_i8";
        case CONV_BF16: return "conv_bf16";
        case CONV3X3_U8_BF16: return "conv3x3_u8";
        case CONV3X3_PATCH: return "conv3x3_patch";
        case CONV3X3_STEM: return "conv3x3_stem";
        case CONV3X3_POOL: return "conv3x3_pool";
        case STEM_POOL: return "stem_pool";
        case CONV_POOL_REGS: return "conv_pool_regs";
        case RES_BLOCK: return "res_block";
        case RES_STAGE: return "res_stage";
        case CONV_IMAGE_BF16: return "conv_image_bf16";
        default: return "generic";
      }
    case OP_POOL: return "pool";
    case OP_FC: return "fc";
    case OP_MEAS: return "meas";
    case OP_GRU: return "rnn";
    case OP_HEADS: return "heads";
  }
  return "";
}

extern "C" int64_t sf_policy_op_flops_per_row(const sf_policy* handle, int i) {
  const Policy* p = reinterpret_cast<const Policy*>(handle);
  if (!p || i < 0 || i >= (int)p->ops.size()) return 0;
  return p->ops[i].flops_per_row;
}

// The arithmetic of launch i, as selected for the current parameters.
extern "C" const char* sf_policy_op_pipe(const sf_policy* handle, int i) {
  const Policy* p = reinterpret_cast<const Policy*>(handle);
  if (!p || i < 0 || i >= (int)p->ops.size()) return "";
  const Op& op = p->ops[i];
  const char* mfma16 = p->act_f16 ? "f16" : "bf16";
  switch (op.kind) {
    case OP_CONV: {
      const ConvLayer& L = p->convs[op.conv];
      switch (L.impl) {
        case CONV1_U8_I8:
          if (op.mid_buf >= 0) return L.planes == 2 ? "i8x2+bf16" : "i8x3+bf16";
          return L.planes == 2 ? "i8x2" : "i8x3";
        case CONV1_U8_MFMA:
        case CONV_GEMM_MFMA: return "f32";
        case CONV_BF16:
        case CONV3X3_PATCH:
        case CONV3X3_STEM:
        case CONV3X3_POOL:
        case STEM_POOL:
        case CONV_POOL_REGS:
        case RES_BLOCK:
        case RES_STAGE:
        case CONV_IMAGE_BF16: return mfma16;
        default: return "valu";
      }
    }
    case OP_FC: return p->fc_wbf ? mfma16 : (p->fc_wt ? "f32" : "valu");
    case OP_GRU: return p->rnn_wih_bf ? "bf16" : (p->gru_wih ? "f32" : "valu");
    default: return "valu";
  }
}

extern "C" double sf_policy_conv1_fixed_point_ratio(const sf_policy* handle, int planes) {
  const Policy* p = reinterpret_cast<const Policy*>(handle);
  if (!p) return -1.0;
  return planes == 2 ? p->conv1_ratio2 : p->conv1_ratio3;
}

// Host only: the admission test on a filter bank [32][cin][8][8], no device involved.
extern "C" int sf_conv1_fixed_point_test(const float* conv_w, int32_t cin, float obs_mul, int32_t dtype,
                                         double* ratio2, double* ratio3) {
  if (!conv_w || !ratio2 || !ratio3 || (cin != 1 && cin != 3 && cin != 4) ||
      (dtype != SF_DTYPE_FP32 && dtype != SF_DTYPE_BF16)) {
    set_error("sf_conv1_fixed_point_test: bad argument");
    return SF_ERR_ARG;
  }
  std::vector<int> ipk;
  std::vector<float> spk, bpk, zero_bias(32, 0.0f);
  Conv1I8Info info;
  conv1_i8_pack(conv_w, zero_bias.data(), cin, 0.0f, obs_mul, dtype == SF_DTYPE_BF16, ipk, spk, bpk, &info);
  *ratio2 = info.ratio2;
  *ratio3 = info.ratio3;
  return SF_OK;
}

extern "C" int sf_policy_set_op_timing(sf_policy* handle, int enable) {
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p) {
    set_error("sf_policy_set_op_timing: null handle");
    return SF_ERR_ARG;
  }
  p->timing = enable != 0;
  return SF_OK;
}

extern "C" int sf_policy_last_op_times(sf_policy* handle, float* ms_out, int n) {
  Policy* p = reinterpret_cast<Policy*>(handle);
  if (!p || !ms_out || n < (int)p->ops.size()) {
    set_error("sf_policy_last_op_times: bad argument");
    return SF_ERR_ARG;
  }
  if (hipEventSynchronize(p->events.back()) != hipSuccess) {
    set_error("sf_policy_last_op_times: no timed step has been recorded");
    return SF_ERR_DEVICE;
  }
  for (size_t i = 0; i < p->ops.size(); ++i)
    if (hipEventElapsedTime(&ms_out[i], p->events[i], p->events[i + 1]) != hipSuccess) {
      set_error("sf_policy_last_op_times: hipEventElapsedTime failed");
      return SF_ERR_DEVICE;
    }
  return SF_OK;
}

extern "C" int sf_copy_bytes(const void* src, void* dst, int64_t bytes, void* hip_stream) {
  if (!src || !dst || bytes < 0 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) {
    set_error("sf_copy_bytes: null or misaligned argument");
    return SF_ERR_ARG;
  }
  hipError_t e = launch_copy16(src, dst, bytes, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) {
    set_error("sf_copy_bytes: launch failed: %s", hipGetErrorString(e));
    return SF_ERR_DEVICE;
  }
  return SF_OK;
}

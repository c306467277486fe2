// Double-buffered stepping (paper, Sec. 3.2): one or two slots of device-side input and
// output buffers around one policy, so that the observations of one half of the
// environments cross the bus while the step of the other half computes.
//
// Three streams, all at the default priority:
//   in   host -> device copies of obs, measurements, done, env_ids
//   cmp  the indexed step (both slots, in submission order: they share the policy's
//        workspace and the state table)
//   out  device -> host copies of actions, logp, value
// and three events per slot chaining them: in -> cmp -> out.  A slot is resubmitted only
// after sf_pipeline_wait, so its buffers are never overwritten while still in use.
#include <vector>

#include "sf_internal.h"

namespace sf {
namespace {

struct Slot {
  uint8_t* obs = nullptr;
  float* meas = nullptr;
  uint8_t* done = nullptr;
  int32_t* ids = nullptr;
  int32_t* actions = nullptr;
  float* logp = nullptr;
  float* value = nullptr;
  hipEvent_t ev_in = nullptr, ev_cmp = nullptr, ev_out = nullptr;
  bool busy = false;
};

struct Pipeline {
  Policy* policy = nullptr;
  int slot_batch = 0;
  size_t obs_row = 0;
  hipStream_t s_in = nullptr, s_cmp = nullptr, s_out = nullptr;
  std::vector<Slot> slots;
};

void free_pipeline(Pipeline* pl) {
  if (!pl) return;
  for (Slot& s : pl->slots) {
    (void)hipFree(s.obs);
    (void)hipFree(s.meas);
    (void)hipFree(s.done);
    (void)hipFree(s.ids);
    (void)hipFree(s.actions);
    (void)hipFree(s.logp);
    (void)hipFree(s.value);
    if (s.ev_in) (void)hipEventDestroy(s.ev_in);
    if (s.ev_cmp) (void)hipEventDestroy(s.ev_cmp);
    if (s.ev_out) (void)hipEventDestroy(s.ev_out);
  }
  if (pl->s_in) (void)hipStreamDestroy(pl->s_in);
  if (pl->s_cmp) (void)hipStreamDestroy(pl->s_cmp);
  if (pl->s_out) (void)hipStreamDestroy(pl->s_out);
  delete pl;
}

}  // namespace
}  // namespace sf

using namespace sf;

#define SF_PL_TRY(expr, code)                                                  \
  do {                                                                         \
    hipError_t e_ = (expr);                                                    \
    if (e_ != hipSuccess) {                                                    \
      set_error("%s: %s failed: %s", fn, #expr, hipGetErrorString(e_));        \
      code;                                                                    \
    }                                                                          \
  } while (0)

extern "C" int sf_pipeline_create(sf_policy* policy, int32_t slot_batch, int32_t n_slots,
                                  sf_pipeline** out) {
  static const char* fn = "sf_pipeline_create";
  if (out) *out = nullptr;
  Policy* p = reinterpret_cast<Policy*>(policy);
  if (!p || !out) {
    set_error("%s: null argument", fn);
    return SF_ERR_ARG;
  }
  if (n_slots != 1 && n_slots != 2) {
    set_error("%s: n_slots = %d, must be 1 or 2", fn, n_slots);
    return SF_ERR_ARG;
  }
  const sf_policy_config& c = p->cfg;
  if (slot_batch < 1 || slot_batch > c.max_batch) {
    set_error("%s: slot_batch = %d outside [1, max_batch = %d]", fn, slot_batch, c.max_batch);
    return SF_ERR_BATCH;
  }
  SF_PL_TRY(hipSetDevice(p->device), return SF_ERR_DEVICE);
  Pipeline* pl = new Pipeline();
  pl->policy = p;
  pl->slot_batch = slot_batch;
  pl->obs_row = (size_t)c.obs_c * c.obs_h * c.obs_w;
  pl->slots.resize(n_slots);
  SF_PL_TRY(hipStreamCreateWithFlags(&pl->s_in, hipStreamNonBlocking), free_pipeline(pl); return SF_ERR_DEVICE);
  SF_PL_TRY(hipStreamCreateWithFlags(&pl->s_cmp, hipStreamNonBlocking), free_pipeline(pl); return SF_ERR_DEVICE);
  SF_PL_TRY(hipStreamCreateWithFlags(&pl->s_out, hipStreamNonBlocking), free_pipeline(pl); return SF_ERR_DEVICE);
  const size_t n = (size_t)slot_batch;
  for (Slot& s : pl->slots) {
    SF_PL_TRY(hipMalloc((void**)&s.obs, n * pl->obs_row), free_pipeline(pl); return SF_ERR_OOM);
    if (c.meas_dim > 0)
      SF_PL_TRY(hipMalloc((void**)&s.meas, n * c.meas_dim * sizeof(float)), free_pipeline(pl);
                return SF_ERR_OOM);
    SF_PL_TRY(hipMalloc((void**)&s.done, n), free_pipeline(pl); return SF_ERR_OOM);
    SF_PL_TRY(hipMalloc((void**)&s.ids, n * sizeof(int32_t)), free_pipeline(pl); return SF_ERR_OOM);
    SF_PL_TRY(hipMalloc((void**)&s.actions, n * c.n_heads * sizeof(int32_t)), free_pipeline(pl);
              return SF_ERR_OOM);
    SF_PL_TRY(hipMalloc((void**)&s.logp, n * sizeof(float)), free_pipeline(pl); return SF_ERR_OOM);
    SF_PL_TRY(hipMalloc((void**)&s.value, n * sizeof(float)), free_pipeline(pl); return SF_ERR_OOM);
    SF_PL_TRY(hipEventCreateWithFlags(&s.ev_in, hipEventDisableTiming), free_pipeline(pl);
              return SF_ERR_DEVICE);
    SF_PL_TRY(hipEventCreateWithFlags(&s.ev_cmp, hipEventDisableTiming), free_pipeline(pl);
              return SF_ERR_DEVICE);
    SF_PL_TRY(hipEventCreateWithFlags(&s.ev_out, hipEventDisableTiming), free_pipeline(pl);
              return SF_ERR_DEVICE);
  }
  *out = reinterpret_cast<sf_pipeline*>(pl);
  return SF_OK;
}

extern "C" int sf_pipeline_submit(sf_pipeline* handle, int32_t slot, int32_t B, const uint8_t* host_obs,
                                  const float* host_meas, const uint8_t* host_done,
                                  const int32_t* host_env_ids,
                                  float* h_table, int32_t n_env, uint64_t seed, uint64_t step,
                                  int32_t* host_actions, float* host_logp, float* host_value) {
  static const char* fn = "sf_pipeline_submit";
  Pipeline* pl = reinterpret_cast<Pipeline*>(handle);
  if (!pl) {
    set_error("%s: null handle", fn);
    return SF_ERR_ARG;
  }
  if (slot < 0 || slot >= (int)pl->slots.size()) {
    set_error("%s: slot %d outside [0, %d)", fn, slot, (int)pl->slots.size());
    return SF_ERR_ARG;
  }
  Slot& s = pl->slots[slot];
  if (s.busy) {
    set_error("%s: slot %d is in flight; call sf_pipeline_wait first", fn, slot);
    return SF_ERR_ARG;
  }
  if (B < 0 || B > pl->slot_batch) {
    set_error("%s: B = %d outside [0, slot_batch = %d]", fn, B, pl->slot_batch);
    return SF_ERR_BATCH;
  }
  if (B == 0) return SF_OK;
  if (!host_obs || !host_done || !host_env_ids || !h_table || !host_actions || !host_logp ||
      !host_value) {
    set_error("%s: null buffer", fn);
    return SF_ERR_ARG;
  }
  const sf_policy_config& c = pl->policy->cfg;
  if (c.meas_dim > 0 && !host_meas) {
    set_error("%s: null measurement buffer", fn);
    return SF_ERR_ARG;
  }
  const size_t n = (size_t)B;
  SF_PL_TRY(hipSetDevice(pl->policy->device), return SF_ERR_DEVICE);
  if (c.meas_dim > 0)
    SF_PL_TRY(hipMemcpyAsync(s.meas, host_meas, n * c.meas_dim * sizeof(float), hipMemcpyHostToDevice,
                             pl->s_in),
              return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(s.obs, host_obs, n * pl->obs_row, hipMemcpyHostToDevice, pl->s_in),
            return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(s.done, host_done, n, hipMemcpyHostToDevice, pl->s_in), return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(s.ids, host_env_ids, n * sizeof(int32_t), hipMemcpyHostToDevice, pl->s_in),
            return SF_ERR_DEVICE);
  SF_PL_TRY(hipEventRecord(s.ev_in, pl->s_in), return SF_ERR_DEVICE);
  SF_PL_TRY(hipStreamWaitEvent(pl->s_cmp, s.ev_in, 0), return SF_ERR_DEVICE);
  int rc = sf_policy_step_indexed(reinterpret_cast<sf_policy*>(pl->policy), B, s.obs, s.meas, h_table, n_env,
                                  s.ids, s.done, seed, step, s.actions, s.logp, s.value, nullptr,
                                  pl->s_cmp);
  if (rc != SF_OK) return rc;
  SF_PL_TRY(hipEventRecord(s.ev_cmp, pl->s_cmp), return SF_ERR_DEVICE);
  SF_PL_TRY(hipStreamWaitEvent(pl->s_out, s.ev_cmp, 0), return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(host_actions, s.actions, n * c.n_heads * sizeof(int32_t),
                           hipMemcpyDeviceToHost, pl->s_out),
            return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(host_logp, s.logp, n * sizeof(float), hipMemcpyDeviceToHost, pl->s_out),
            return SF_ERR_DEVICE);
  SF_PL_TRY(hipMemcpyAsync(host_value, s.value, n * sizeof(float), hipMemcpyDeviceToHost, pl->s_out),
            return SF_ERR_DEVICE);
  SF_PL_TRY(hipEventRecord(s.ev_out, pl->s_out), return SF_ERR_DEVICE);
  s.busy = true;
  return SF_OK;
}

extern "C" int sf_pipeline_wait(sf_pipeline* handle, int32_t slot) {
  static const char* fn = "sf_pipeline_wait";
  Pipeline* pl = reinterpret_cast<Pipeline*>(handle);
  if (!pl) {
    set_error("%s: null handle", fn);
    return SF_ERR_ARG;
  }
  if (slot < 0 || slot >= (int)pl->slots.size()) {
    set_error("%s: slot %d outside [0, %d)", fn, slot, (int)pl->slots.size());
    return SF_ERR_ARG;
  }
  Slot& s = pl->slots[slot];
  if (!s.busy) return SF_OK;
  SF_PL_TRY(hipEventSynchronize(s.ev_out), return SF_ERR_DEVICE);
  s.busy = false;
  return SF_OK;
}

extern "C" int sf_pipeline_destroy(sf_pipeline* handle) {
  Pipeline* pl = reinterpret_cast<Pipeline*>(handle);
  if (!pl) return SF_OK;
  int rc = SF_OK;
  for (Slot& s : pl->slots)
    if (s.busy && hipEventSynchronize(s.ev_out) != hipSuccess) rc = SF_ERR_DEVICE;
  free_pipeline(pl);
  return rc;
}

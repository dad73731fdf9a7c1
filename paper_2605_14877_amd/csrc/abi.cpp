// extern "C" entry points of libheatkv: argument checks, plan life cycle, and
// the hand-off to the kernel launchers.  No arithmetic of the method lives here.
#include <cstdint>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "heatkv.h"
#include "kernels.h"
#include "plan.h"

namespace heatkv {
const char* last_error_cstr();
}

using heatkv::fail;

namespace {

int hip_fail(hipError_t e, const char* what) {
  return fail(HEATKV_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

void free_device(heatkv::DeviceTables& d) {
  if (d.block) (void)hipFree(d.block);
  d = heatkv::DeviceTables{};
}

// One device allocation and one copy for all plan tables (16-byte aligned sections).
int ensure_uploaded(heatkv_plan* p) {
  std::lock_guard<std::mutex> lock(p->upload_mutex);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (p->dev.device == dev) return HEATKV_OK;
  if (p->dev.device >= 0) return fail(HEATKV_EINVAL, "plan was uploaded to another device");
  auto pad = [](size_t n) { return (n + 15) / 16 * 16; };
  const size_t nw = p->run_row.size() * sizeof(heatkv::HeadWork);
  const size_t nd = p->descs.size() * sizeof(heatkv::CopyDesc);
  const size_t o_work = 0, o_desc = o_work + pad(nw);
  const size_t total = o_desc + pad(nd) + 16;
  std::vector<unsigned char> host;
  try {
    host.assign(total, 0);
  } catch (const std::bad_alloc&) {
    return fail(HEATKV_ENOMEM, "out of host memory");
  }
  {  // per (scale, layer): the heads in the order of head_order, each with its run
    heatkv::HeadWork* w = reinterpret_cast<heatkv::HeadWork*>(host.data() + o_work);
    const size_t groups = p->run_row.size() / size_t(p->H);
    for (size_t g = 0; g < groups; ++g)
      for (int r = 0; r < p->H; ++r) {
        const int32_t h = p->head_order[g * p->H + r];
        w[g * p->H + r] = heatkv::HeadWork{h, p->run_row[g * p->H + h], p->run_len[g * p->H + h], 0};
      }
  }
  if (nd) std::memcpy(host.data() + o_desc, p->descs.data(), nd);
  void* block = nullptr;
  e = hipMalloc(&block, total);
  if (e != hipSuccess) return fail(HEATKV_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  e = hipMemcpy(block, host.data(), total, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(block);
    return hip_fail(e, "hipMemcpy");
  }
  // Everything a launch may need to set up on this device happens here, not at the first launch, so that the
  // launches themselves only enqueue kernels (a caller may be capturing them into a graph).
  if (p->dtype == HEATKV_BF16) {
    e = heatkv::attend_prepare_device();
    if (e != hipSuccess) {
      (void)hipFree(block);
      return hip_fail(e, "attention kernel set-up");
    }
  }
  unsigned char* base = static_cast<unsigned char*>(block);
  p->dev.block = block;
  p->dev.work = reinterpret_cast<heatkv::HeadWork*>(base + o_work);
  p->dev.descs = reinterpret_cast<heatkv::CopyDesc*>(base + o_desc);
  p->dev.device = dev;
  return HEATKV_OK;
}

int check_plan_index(const heatkv_plan* p, int layer, int k) {
  if (!p) return fail(HEATKV_EINVAL, "plan is null");
  if (layer < 0 || layer >= p->L) return fail(HEATKV_EINVAL, "layer out of range");
  if (k < 0 || k >= p->K) return fail(HEATKV_EINVAL, "scale index out of range");
  return HEATKV_OK;
}

// 8-bit cache rows exist for the matrix-core attention path only (bf16, d = 128).
int check_kv_format(const heatkv_plan* p, int kv_format) {
  if (kv_format == HEATKV_KV_NATIVE) return HEATKV_OK;
  if (kv_format != HEATKV_KV_FP8_E4M3) return fail(HEATKV_EINVAL, "unknown cache storage format");
  if (p->dtype != HEATKV_BF16 || p->d != 128)
    return fail(HEATKV_EINVAL, "HEATKV_KV_FP8_E4M3 needs a bf16 shape with head dimension 128");
  return HEATKV_OK;
}

int finish_plan(heatkv_plan* p, heatkv_plan** out) {
  int rc = heatkv::derive_layout(p);
  if (rc) {
    delete p;
    return rc;
  }
  *out = p;
  return HEATKV_OK;
}

}  // namespace

extern "C" {

const char* heatkv_last_error(void) { return heatkv::last_error_cstr(); }

int heatkv_build_schedule_kv(const heatkv_shape* shape, const float* beta, uint64_t budget_bytes_per_seq, int sinks,
                             int variant, int kv_format, heatkv_plan** out) {
  if (!out) return fail(HEATKV_EINVAL, "out is null");
  *out = nullptr;
  if (!beta) return fail(HEATKV_EINVAL, "beta is null");
  if (variant < 0 || variant > 3) return fail(HEATKV_EINVAL, "unknown variant");
  heatkv_plan* p = new (std::nothrow) heatkv_plan;
  if (!p) return fail(HEATKV_ENOMEM, "out of host memory");
  int rc = heatkv::init_shape(p, shape);
  if (!rc && (sinks < 0 || sinks > p->K - 2)) rc = fail(HEATKV_EINVAL, "sinks must be in [0, K-2]");
  if (!rc) rc = check_kv_format(p, kv_format);
  if (rc) {
    delete p;
    return rc;
  }
  p->sinks = sinks;
  p->variant = variant;
  p->from_schedule = true;
  p->kv_format = kv_format;
  p->B = int64_t(budget_bytes_per_seq / (2u * uint64_t(p->d) * p->kv_elem_size()));
  try {
    rc = heatkv::build_sets(p, beta);
    if (rc) {
      delete p;
      return rc;
    }
    return finish_plan(p, out);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(HEATKV_ENOMEM, "out of host memory");
  }
}

int heatkv_build_schedule(const heatkv_shape* shape, const float* beta, uint64_t budget_bytes_per_seq, int sinks,
                          int variant, heatkv_plan** out) {
  return heatkv_build_schedule_kv(shape, beta, budget_bytes_per_seq, sinks, variant, HEATKV_KV_NATIVE, out);
}

int heatkv_load_schedule_kv(const heatkv_shape* shape, const uint8_t* present, int kv_format, heatkv_plan** out) {
  if (!out) return fail(HEATKV_EINVAL, "out is null");
  *out = nullptr;
  if (!present) return fail(HEATKV_EINVAL, "present is null");
  heatkv_plan* p = new (std::nothrow) heatkv_plan;
  if (!p) return fail(HEATKV_ENOMEM, "out of host memory");
  int rc = heatkv::init_shape(p, shape);
  if (!rc) rc = check_kv_format(p, kv_format);
  if (rc) {
    delete p;
    return rc;
  }
  p->kv_format = kv_format;
  try {
    rc = heatkv::load_pattern(p, present);
    if (rc) {
      delete p;
      return rc;
    }
    return finish_plan(p, out);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(HEATKV_ENOMEM, "out of host memory");
  }
}

int heatkv_load_schedule(const heatkv_shape* shape, const uint8_t* present, heatkv_plan** out) {
  return heatkv_load_schedule_kv(shape, present, HEATKV_KV_NATIVE, out);
}

int heatkv_plan_kv_format(const heatkv_plan* plan) { return plan ? plan->kv_format : HEATKV_KV_NATIVE; }

void heatkv_plan_destroy(heatkv_plan* plan) {
  if (!plan) return;
  if (plan->dev.device >= 0) free_device(plan->dev);
  delete plan;
}

int heatkv_plan_upload(heatkv_plan* plan) {
  if (!plan) return fail(HEATKV_EINVAL, "plan is null");
  return ensure_uploaded(plan);
}

int64_t heatkv_plan_budget_tokens(const heatkv_plan* plan) { return plan ? plan->B : 0; }

int heatkv_plan_N(const heatkv_plan* plan, int32_t* out) {
  if (!plan || !out) return fail(HEATKV_EINVAL, "null argument");
  if (!plan->from_schedule) return fail(HEATKV_EINVAL, "plan was loaded from an explicit pattern");
  std::memcpy(out, plan->N.data(), plan->N.size() * sizeof(int32_t));
  return HEATKV_OK;
}

int heatkv_plan_order(const heatkv_plan* plan, int i, int32_t* heads_out) {
  if (!plan || !heads_out) return fail(HEATKV_EINVAL, "null argument");
  if (!plan->from_schedule) return fail(HEATKV_EINVAL, "plan was loaded from an explicit pattern");
  if (i < plan->sinks || i >= plan->K - 1) return fail(HEATKV_EINVAL, "source scale has no order");
  std::memcpy(heads_out, plan->orders[i].data(), size_t(plan->T) * sizeof(int32_t));
  return HEATKV_OK;
}

int heatkv_plan_sets(const heatkv_plan* plan, int k, int which, uint8_t* bitmap) {
  if (!plan || !bitmap) return fail(HEATKV_EINVAL, "null argument");
  if (!plan->from_schedule) return fail(HEATKV_EINVAL, "plan was loaded from an explicit pattern");
  const int kmax = which == HEATKV_SET_A ? plan->K : plan->K - 1;
  if (k < 0 || k >= kmax) return fail(HEATKV_EINVAL, "scale index out of range");
  const std::vector<uint8_t>* src = which == HEATKV_SET_G ? &plan->G : which == HEATKV_SET_E ? &plan->E
                                    : which == HEATKV_SET_A ? &plan->A : nullptr;
  if (!src) return fail(HEATKV_EINVAL, "unknown set");
  const size_t KT = size_t(plan->K) * plan->T;
  std::memcpy(bitmap, src->data() + size_t(k) * KT, KT);
  return HEATKV_OK;
}

int heatkv_plan_retained(const heatkv_plan* plan, int k, int layer, int head, int32_t* token_idx, int32_t* n) {
  int rc = check_plan_index(plan, layer, k);
  if (rc) return rc;
  if (!n) return fail(HEATKV_EINVAL, "n is null");
  if (head < 0 || head >= plan->H) return fail(HEATKV_EINVAL, "head out of range");
  const uint32_t m = plan->retained[size_t(k) * plan->T + layer * plan->H + head];
  int32_t cnt = 0;
  for (int i = 0; i < k; ++i) {
    if (!(m >> i & 1u)) continue;
    const int32_t lo = plan->c[i] - plan->t[i];
    if (token_idx)
      for (int32_t j = 0; j < plan->t[i]; ++j) token_idx[cnt + j] = lo + j;
    cnt += plan->t[i];
  }
  *n = cnt;
  return HEATKV_OK;
}

int64_t heatkv_plan_arena_tokens(const heatkv_plan* plan) { return plan ? plan->arena_tokens : 0; }

size_t heatkv_plan_arena_bytes(const heatkv_plan* plan) {
  if (!plan) return 0;
  return size_t(plan->batch) * size_t(plan->arena_tokens) * size_t(plan->d) * plan->kv_elem_size();
}

int heatkv_plan_runs(const heatkv_plan* plan, int k, int layer, int32_t* row_out, int32_t* len_out) {
  int rc = check_plan_index(plan, layer, k);
  if (rc) return rc;
  if (!row_out || !len_out) return fail(HEATKV_EINVAL, "null argument");
  std::memcpy(row_out, &plan->run_row[plan->idx(k, layer, 0)], size_t(plan->H) * sizeof(int32_t));
  std::memcpy(len_out, &plan->run_len[plan->idx(k, layer, 0)], size_t(plan->H) * sizeof(int32_t));
  return HEATKV_OK;
}

int64_t heatkv_plan_live_tokens(const heatkv_plan* plan, int k, int layer) {
  if (check_plan_index(plan, layer, k)) return -1;
  if (k >= plan->K - 1) return -1;
  int64_t live = 0;
  for (int l = 0; l < plan->L; ++l) live += plan->region_size[plan->idx(l <= layer ? k + 1 : k, l)];
  return live;
}

int heatkv_append_scale(heatkv_plan* plan, int layer, int k, const void* k_new, const void* v_new, void* k_arena,
                        void* v_arena, void* stream) {
  int rc = check_plan_index(plan, layer, k);
  if (rc) return rc;
  if (k == plan->K - 1) return HEATKV_OK;
  if (!k_new || !v_new || !k_arena || !v_arena) return fail(HEATKV_EINVAL, "null tensor pointer");
  const int ndesc = plan->desc_count[plan->idx(k, layer)];
  if (ndesc == 0) return HEATKV_OK;
  if ((rc = ensure_uploaded(plan))) return rc;
  heatkv::AppendArgs a{};
  a.row_bytes = int(plan->d * plan->elem_size());
  a.kv_fp8 = plan->kv_format == HEATKV_KV_FP8_E4M3;
  a.batch = plan->batch;
  a.H = plan->H;
  a.t_k = plan->t[k];
  a.arena_tokens = plan->arena_tokens;
  a.descs = plan->dev.descs + plan->desc_begin[plan->idx(k, layer)];
  a.ndesc = ndesc;
  a.k_new = k_new;
  a.v_new = v_new;
  a.k_arena = k_arena;
  a.v_arena = v_arena;
  hipError_t e = heatkv::launch_append(a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "append_scale launch");
  return HEATKV_OK;
}

size_t heatkv_attend_workspace_bytes(const heatkv_plan* plan, int layer, int k) {
  if (check_plan_index(plan, layer, k)) return 0;
  return heatkv::attend_workspace_bytes(plan->dtype, plan->d, plan->H, plan->batch, plan->t[k],
                                        plan->max_len[plan->idx(k, layer)]);
}

namespace {

// Shared body of heatkv_attend_scale and heatkv_attend_append_scale.
int attend_impl(heatkv_plan* plan, int layer, int k, const void* q, const void* k_cur, const void* v_cur,
                const void* k_arena, const void* v_arena, void* k_arena_rw, void* v_arena_rw, bool with_append,
                float sm_scale, void* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_plan_index(plan, layer, k);
  if (rc) return rc;
  if (!q || !k_cur || !v_cur || !out) return fail(HEATKV_EINVAL, "null tensor pointer");
  const int max_len = plan->max_len[plan->idx(k, layer)];
  if (max_len > 0 && (!k_arena || !v_arena)) return fail(HEATKV_EINVAL, "null arena pointer");
  const size_t need = heatkv::attend_workspace_bytes(plan->dtype, plan->d, plan->H, plan->batch, plan->t[k], max_len);
  if (need > 0 && (!ws || ws_bytes < need)) return fail(HEATKV_EINVAL, "attend workspace too small");
  const int ndesc = (with_append && k < plan->K - 1) ? plan->desc_count[plan->idx(k, layer)] : 0;
  if (ndesc > 0 && (!k_arena_rw || !v_arena_rw)) return fail(HEATKV_EINVAL, "null arena pointer");
  if ((rc = ensure_uploaded(plan))) return rc;
  heatkv::AttendArgs a{};
  a.dtype = plan->dtype;
  a.kv_fp8 = plan->kv_format == HEATKV_KV_FP8_E4M3;
  a.d = plan->d;
  a.H = plan->H;
  a.batch = plan->batch;
  a.t_k = plan->t[k];
  a.arena_tokens = plan->arena_tokens;
  const size_t off = plan->idx(k, layer, 0);
  a.work = plan->dev.work + off;
  a.max_len = max_len;
  {  // runs of equal length (no head of the layer has lost a scale yet): addresses follow from the head index
    const int32_t* len = &plan->run_len[off];
    bool uniform = true;
    for (int h = 1; h < plan->H; ++h) uniform = uniform && len[h] == len[0];
    if (uniform) {
      a.uniform_len = len[0];
      a.uniform_row0 = plan->run_row[off];
    }
  }
  a.q = q;
  a.k_cur = k_cur;
  a.v_cur = v_cur;
  a.k_arena = k_arena;
  a.v_arena = v_arena;
  a.out = out;
  a.sm_scale = sm_scale;
  a.ws = ws;
  a.ws_bytes = ws_bytes;
  if (ndesc > 0) {
    a.descs = plan->dev.descs + plan->desc_begin[plan->idx(k, layer)];
    a.ndesc = ndesc;
    a.row_bytes = int(plan->d * plan->elem_size());
    a.k_arena_rw = k_arena_rw;
    a.v_arena_rw = v_arena_rw;
  }
  hipError_t e = heatkv::launch_attend(a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "attend_scale launch");
  return HEATKV_OK;
}

}  // namespace

int heatkv_attend_scale(heatkv_plan* plan, int layer, int k, const void* q, const void* k_cur, const void* v_cur,
                        const void* k_arena, const void* v_arena, float sm_scale, void* out, void* ws,
                        size_t ws_bytes, void* stream) {
  return attend_impl(plan, layer, k, q, k_cur, v_cur, k_arena, v_arena, nullptr, nullptr, false, sm_scale, out, ws,
                     ws_bytes, stream);
}

int heatkv_attend_append_scale(heatkv_plan* plan, int layer, int k, const void* q, const void* k_cur,
                               const void* v_cur, void* k_arena, void* v_arena, float sm_scale, void* out, void* ws,
                               size_t ws_bytes, void* stream) {
  return attend_impl(plan, layer, k, q, k_cur, v_cur, k_arena, v_arena, k_arena, v_arena, true, sm_scale, out, ws,
                     ws_bytes, stream);
}

size_t heatkv_calibrate_workspace_bytes(const heatkv_shape* shape, int k1) {
  if (heatkv::check_shape(shape)) return 0;
  if (k1 < 0 || k1 >= shape->K) return 0;
  return heatkv::calibrate_workspace_bytes(shape->dtype, shape->d, shape->H, shape->batch, shape->K, shape->t[k1]);
}

namespace {

int calibrate_impl(const heatkv_shape* shape, int layer, int n_scales, const int32_t* k1, const void* const* q,
                   const void* const* k_all, float sm_scale, float* const* mass, float weight, float* beta, void* ws,
                   size_t ws_bytes, void* stream) {
  int rc = heatkv::check_shape(shape);
  if (rc) return rc;
  if (layer < 0 || layer >= shape->L) return fail(HEATKV_EINVAL, "layer out of range");
  if (n_scales < 1 || n_scales > shape->K) return fail(HEATKV_EINVAL, "number of scales out of range");
  if (!k1 || !q || !k_all) return fail(HEATKV_EINVAL, "null argument array");
  heatkv::CalibrateArgs a{};
  bool seen[HEATKV_MAX_SCALES] = {};
  for (int i = 0; i < n_scales; ++i) {
    if (k1[i] < 0 || k1[i] >= shape->K) return fail(HEATKV_EINVAL, "scale index out of range");
    if (seen[k1[i]]) return fail(HEATKV_EINVAL, "scale listed twice");
    seen[k1[i]] = true;
    float* m = mass ? mass[i] : nullptr;
    if (!q[i] || !k_all[i] || (!m && !beta)) return fail(HEATKV_EINVAL, "null tensor pointer");
    a.k1[i] = k1[i];
    a.q[i] = q[i];
    a.k_all[i] = k_all[i];
    a.mass[i] = m;
  }
  const size_t need = heatkv::calibrate_scales_workspace_bytes(shape->dtype, shape->d, shape->H, shape->batch, shape->K,
                                                               shape->t, n_scales, k1);
  // a single scale needs no padding between scales: the exact size is enough there
  const size_t need_single =
      heatkv::calibrate_workspace_bytes(shape->dtype, shape->d, shape->H, shape->batch, shape->K, shape->t[k1[0]]);
  if (!ws || ws_bytes < (n_scales == 1 ? need_single : need))
    return fail(HEATKV_EINVAL, "calibrate workspace too small");
  if (reinterpret_cast<uintptr_t>(ws) % 4 != 0) return fail(HEATKV_EINVAL, "calibrate workspace must be 4-byte aligned");
  a.dtype = shape->dtype;
  a.d = shape->d;
  a.H = shape->H;
  a.batch = shape->batch;
  a.K = shape->K;
  a.n_scales = n_scales;
  for (int k = 0; k < shape->K; ++k) a.t[k] = shape->t[k];
  a.sm_scale = sm_scale;
  a.ws = ws;
  a.beta = beta;
  a.weight = weight;
  a.layer = layer;
  hipError_t e = heatkv::launch_calibrate(a, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "calibrate launch");
  return HEATKV_OK;
}

}  // namespace

int heatkv_calibrate(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all, float sm_scale,
                     float* mass, void* ws, size_t ws_bytes, void* stream) {
  if (!mass) return fail(HEATKV_EINVAL, "null tensor pointer");
  const int32_t k = k1;
  return calibrate_impl(shape, layer, 1, &k, &q, &k_all, sm_scale, &mass, 0.f, nullptr, ws, ws_bytes, stream);
}

int heatkv_calibrate_static(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all,
                            float sm_scale, float* mass, void* stream) {
  if (!mass) return fail(HEATKV_EINVAL, "null tensor pointer");
  // size first: a shape that does not fit is refused before any HIP call
  const size_t need = heatkv_calibrate_workspace_bytes(shape, k1);
  if (need > heatkv::kCalibrateStaticBytes)
    return fail(HEATKV_EINVAL, "calibrate_static: batch*H*ceil(t[k1]/128)*K*4 = " + std::to_string(need) +
                                   " bytes of partial sums exceed the static workspace of " +
                                   std::to_string(heatkv::kCalibrateStaticBytes) + " bytes; use heatkv_calibrate");
  int rc = heatkv::check_shape(shape);
  if (rc) return rc;
  if (k1 < 0 || k1 >= shape->K) return fail(HEATKV_EINVAL, "scale index out of range");
  void* ws = nullptr;
  hipError_t e = heatkv::calibrate_static_workspace(&ws);
  if (e != hipSuccess) return hip_fail(e, "static workspace lookup");
  const int32_t k = k1;
  return calibrate_impl(shape, layer, 1, &k, &q, &k_all, sm_scale, &mass, 0.f, nullptr, ws,
                        heatkv::kCalibrateStaticBytes, stream);
}

int heatkv_calibrate_accumulate(const heatkv_shape* shape, int layer, int k1, const void* q, const void* k_all,
                                float sm_scale, float weight, float* beta, float* mass, void* ws, size_t ws_bytes,
                                void* stream) {
  if (!beta) return fail(HEATKV_EINVAL, "null tensor pointer");
  const int32_t k = k1;
  return calibrate_impl(shape, layer, 1, &k, &q, &k_all, sm_scale, &mass, weight, beta, ws, ws_bytes, stream);
}

size_t heatkv_calibrate_scales_workspace_bytes(const heatkv_shape* shape, int n_scales, const int32_t* k1) {
  if (heatkv::check_shape(shape) || !k1 || n_scales < 1 || n_scales > shape->K) return 0;
  for (int i = 0; i < n_scales; ++i)
    if (k1[i] < 0 || k1[i] >= shape->K) return 0;
  return heatkv::calibrate_scales_workspace_bytes(shape->dtype, shape->d, shape->H, shape->batch, shape->K, shape->t,
                                                  n_scales, k1);
}

int heatkv_calibrate_scales_accumulate(const heatkv_shape* shape, int layer, int n_scales, const int32_t* k1,
                                       const void* const* q, const void* const* k_all, float sm_scale, float weight,
                                       float* beta, float* const* mass, void* ws, size_t ws_bytes, void* stream) {
  if (!beta) return fail(HEATKV_EINVAL, "null tensor pointer");
  return calibrate_impl(shape, layer, n_scales, k1, q, k_all, sm_scale, mass, weight, beta, ws, ws_bytes, stream);
}

int heatkv_accumulate_beta(const heatkv_shape* shape, int layer, int k1, const float* mass, float weight, float* beta,
                           void* stream) {
  int rc = heatkv::check_shape(shape);
  if (rc) return rc;
  if (layer < 0 || layer >= shape->L) return fail(HEATKV_EINVAL, "layer out of range");
  if (k1 < 0 || k1 >= shape->K) return fail(HEATKV_EINVAL, "scale index out of range");
  if (!mass || !beta) return fail(HEATKV_EINVAL, "null tensor pointer");
  hipError_t e = heatkv::launch_accumulate_beta(shape->H, shape->batch, shape->K, layer, k1, mass, weight, beta,
                                                static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "accumulate_beta launch");
  return HEATKV_OK;
}

int heatkv_head_scores(const heatkv_shape* shape, const float* beta, int sinks, int variant, double* scores) {
  try {
    return heatkv::rank_scores(shape, beta, sinks, variant, scores);
  } catch (const std::bad_alloc&) {
    return fail(HEATKV_ENOMEM, "out of host memory");
  }
}

int heatkv_rank_dispersion(const heatkv_shape* shape, const float* betas, int runs, int sinks, int variant,
                           double* dispersion) {
  try {
    return heatkv::rank_dispersion(shape, betas, runs, sinks, variant, dispersion);
  } catch (const std::bad_alloc&) {
    return fail(HEATKV_ENOMEM, "out of host memory");
  }
}

}  // extern "C"

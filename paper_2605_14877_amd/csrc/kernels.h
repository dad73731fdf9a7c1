// Launchers of the HIP kernels behind the C ABI.  Each returns a hipError_t as int.
#pragma once

#include <cstddef>
#include <cstdint>

#include <hip/hip_runtime_api.h>

#include "plan.h"

namespace heatkv {

struct AttendArgs {
  int dtype, d, H, batch;
  bool kv_fp8 = false;       // arena rows are FP8 E4M3 codes (d bytes per row) instead of the dtype's
  int t_k;                   // queries (= current-scale keys) per head
  int64_t arena_tokens;      // rows per batch entry of each arena
  const HeadWork* work;      // device [H]: the layer's heads by descending run length, each with its run
  int max_len;               // longest run among the H heads (host copy)
  int uniform_len = -1;      // >= 0: all H runs have this length and lie back to back from row uniform_row0 in
  int uniform_row0 = 0;      //       head order; the bf16 kernel then needs no table read (the fp32 one ignores it)
  const void *q, *k_cur, *v_cur, *k_arena, *v_arena;
  void* out;
  float sm_scale;
  void* ws;
  size_t ws_bytes;
  // Optional fused cache update (append_scale of the same layer and scale): extra workgroups of the same
  // launch run these copy descriptors.  ndesc == 0: attention only.
  const CopyDesc* descs = nullptr;
  int ndesc = 0;
  int row_bytes = 0;
  void *k_arena_rw = nullptr, *v_arena_rw = nullptr;
};

size_t attend_workspace_bytes(int dtype, int d, int H, int batch, int t_k, int max_len);
hipError_t launch_attend(const AttendArgs& a, hipStream_t stream);

struct AppendArgs {
  int row_bytes;             // d * elem_size of the new scale's tensors
  bool kv_fp8 = false;       // arena rows are FP8 E4M3 codes: rows from the new scale are converted on the way in
  int batch, H, t_k;
  int64_t arena_tokens;
  const CopyDesc* descs;     // device
  int ndesc;
  const void *k_new, *v_new;
  void *k_arena, *v_arena;
};
hipError_t launch_append(const AppendArgs& a, hipStream_t stream);

struct CalibrateArgs {
  int dtype, d, H, batch, K;
  int32_t t[HEATKV_MAX_SCALES];
  // One launch covers n_scales query scales (distinct k1); entry i reads q[i] and k_all[i] and, if mass[i] is
  // set, writes the per-row masses there.
  int n_scales = 0;
  int32_t k1[HEATKV_MAX_SCALES];
  const void* q[HEATKV_MAX_SCALES];
  const void* k_all[HEATKV_MAX_SCALES];
  float* mass[HEATKV_MAX_SCALES];
  float sm_scale;
  void* ws;  // calibrate_scales_workspace_bytes(...) bytes, 256-byte aligned
  // Optional fused dataset average: beta[layer][h][k1][:] += weight * sum_b mass[b][h][:] (mass may then be null).
  float* beta = nullptr;
  float weight = 0.f;
  int layer = 0;
};
size_t calibrate_workspace_bytes(int dtype, int d, int H, int batch, int K, int t_k1);
size_t calibrate_scales_workspace_bytes(int dtype, int d, int H, int batch, int K, const int32_t* t, int n_scales,
                                        const int32_t* k1);
hipError_t launch_calibrate(const CalibrateArgs& a, hipStream_t stream);
// The library's own calibrate workspace on the current device: a static device array of kCalibrateStaticBytes
// (looked up once per device, no allocation).  Calls that use it on one GPU share it.
constexpr size_t kCalibrateStaticBytes = size_t(1) << 20;
hipError_t calibrate_static_workspace(void** ptr);
// beta[(layer*H + h)*K*K + k1*K + k2] += weight * sum_b mass[(b*H + h)*K + k2]
hipError_t launch_accumulate_beta(int H, int batch, int K, int layer, int k1, const float* mass, float weight,
                                  float* beta, hipStream_t stream);

// One-time set-up of the attention kernels on the current device (the LDS limit of the two-stream instance);
// called at plan upload, repeated calls are cheap.
hipError_t attend_prepare_device();

}  // namespace heatkv

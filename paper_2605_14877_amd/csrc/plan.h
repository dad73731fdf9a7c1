// Internal layout of a heatkv_plan: the static pruning schedule (Sec. 3.3,
// Alg. 1) and everything the kernels derive from it ahead of time.
#pragma once

#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "heatkv.h"

namespace heatkv {

// One contiguous block of rows moved by append_scale.  src_kind 0: rows come
// from the arena (src_row is an arena row of the same batch entry); 1: rows
// come from the new scale's tensor (src_row = head * t[k] + token).
struct CopyDesc {
  int32_t dst_row;
  int32_t src_row;
  int32_t nrows;
  int32_t src_kind;
};

// What an attention workgroup needs to know about its head, one 16-byte record per (scale, layer, rank):
// rank 0 is the head with the longest retained run (workgroups are dealt out longest first).
struct HeadWork {
  int32_t head;     // head index within the layer
  int32_t run_row;  // first arena row of the head's run (per batch entry)
  int32_t run_len;  // retained prior tokens
  int32_t pad;
};

struct DeviceTables {
  int device = -1;
  void* block = nullptr;      // one allocation holding the two tables below
  HeadWork* work = nullptr;   // [K][L][H], by rank
  CopyDesc* descs = nullptr;  // all append descriptors, back to back
};

}  // namespace heatkv

struct heatkv_plan {
  // shape
  int32_t L = 0, H = 0, d = 0, K = 0, batch = 0, dtype = 0, sinks = 0, variant = 0;
  int32_t kv_format = HEATKV_KV_NATIVE;  // how the arenas store a row
  int32_t T = 0;
  bool from_schedule = false;  // false: built from an explicit retention pattern
  std::vector<int32_t> t, c;   // c[k] = t[0]+..+t[k]
  int64_t B = 0;               // token budget (Alg. 1, first line)

  // schedule (only when from_schedule)
  std::vector<int32_t> N;                    // [K-1]
  std::vector<std::vector<int32_t>> orders;  // [K] (valid for i in [sinks,K-1)), each [T]
  std::vector<uint8_t> G, E, A;              // [K][K][T]: set of scale k, source scale i, head

  // retained[k*T + head]: bit i set iff prior scale i (< k) is attended at scale k
  std::vector<uint32_t> retained;

  // physical layout
  std::vector<int32_t> run_len;      // [K][L][H]
  std::vector<int32_t> run_row;      // [K][L][H] absolute arena row (per batch entry)
  std::vector<int32_t> head_order;   // [K][L][H]
  std::vector<int64_t> region_size;  // [K][L] rows of layer l's region at scale k
  std::vector<int64_t> region_base;  // [K][L]
  std::vector<int32_t> max_len;      // [K][L] longest run
  int64_t arena_tokens = 0;

  std::vector<heatkv::CopyDesc> descs;
  std::vector<int64_t> desc_begin;  // [K][L] index into descs
  std::vector<int32_t> desc_count;  // [K][L]

  std::mutex upload_mutex;
  heatkv::DeviceTables dev;

  size_t elem_size() const { return dtype == HEATKV_BF16 ? 2 : 4; }
  size_t kv_elem_size() const { return kv_format == HEATKV_KV_FP8_E4M3 ? 1 : elem_size(); }
  size_t idx(int k, int l, int h) const { return (static_cast<size_t>(k) * L + l) * H + h; }
  size_t idx(int k, int l) const { return static_cast<size_t>(k) * L + l; }
};

namespace heatkv {

void set_error(const std::string& msg);
int fail(int code, const std::string& msg);

// Validates a shape; on success fills the plan's shape fields, t and c.
int init_shape(heatkv_plan* p, const heatkv_shape* shape);
int check_shape(const heatkv_shape* shape);

// Alg. 1 (+ Eq. 3-5): fills N, orders, G, E, A and `retained`.
int build_sets(heatkv_plan* p, const float* beta);
// Head scores behind the orders (Eq. 3 / Eq. 4, un-normalised) and the dispersion of the rank positions
// over several calibration runs (App. C); host only, no plan involved.
int rank_scores(const heatkv_shape* shape, const float* beta, int sinks, int variant, double* scores);
int rank_dispersion(const heatkv_shape* shape, const float* betas, int runs, int sinks, int variant,
                    double* dispersion);
// Fills `retained` from an explicit pattern.
int load_pattern(heatkv_plan* p, const uint8_t* present);
// Derives run tables, the FIFO arena placement and the append descriptors from `retained`.
int derive_layout(heatkv_plan* p);

}  // namespace heatkv

// Descriptor-driven row copy shared by the append kernel and by the attention kernels' fused append blocks.
#pragma once

#include "device_util.h"
#include "plan.h"

namespace heatkv {

struct CopyParams {
  int chunks_per_row;  // row_bytes / 16
  int H, t_k;
  long long arena_tokens;
  const CopyDesc* descs;
  const uint4 *k_new, *v_new;
  uint4 *k_arena, *v_arena;
};

// One workgroup (256 lanes) moves descriptor `desc` of batch entry `b`: up to 128 contiguous rows, 16 bytes per
// lane, four independent loads in flight per lane and arena, K and V together.  Source and destination never
// overlap (the planner places the new region of a layer in free space).
__device__ __forceinline__ void copy_rows_block(const CopyParams& p, int desc, int b) {
  const CopyDesc d = p.descs[desc];
  const long long cpr = p.chunks_per_row;
  const long long arena_base = static_cast<long long>(b) * p.arena_tokens * cpr;
  const long long dst0 = arena_base + static_cast<long long>(d.dst_row) * cpr;
  const uint4 *ks, *vs;
  if (d.src_kind == 0) {
    const long long s0 = arena_base + static_cast<long long>(d.src_row) * cpr;
    ks = p.k_arena + s0;
    vs = p.v_arena + s0;
  } else {
    const long long s0 = (static_cast<long long>(b) * p.H * p.t_k + d.src_row) * cpr;
    ks = p.k_new + s0;
    vs = p.v_new + s0;
  }
  uint4* kd = p.k_arena + dst0;
  uint4* vd = p.v_arena + dst0;
  const int total = d.nrows * p.chunks_per_row;
  // Whole groups of 4 x 256 chunks take the unconditional path (eight loads in flight per lane, all values
  // in registers); the remainder goes one chunk per lane at a time.
  const int whole = total & ~1023;
  for (int i = threadIdx.x; i < whole; i += 4 * 256) {
    const uint4 k0 = ks[i], k1 = ks[i + 256], k2 = ks[i + 512], k3 = ks[i + 768];
    const uint4 v0 = vs[i], v1 = vs[i + 256], v2 = vs[i + 512], v3 = vs[i + 768];
    kd[i] = k0;
    kd[i + 256] = k1;
    kd[i + 512] = k2;
    kd[i + 768] = k3;
    vd[i] = v0;
    vd[i + 256] = v1;
    vd[i + 512] = v2;
    vd[i + 768] = v3;
  }
  for (int i = whole + threadIdx.x; i < total; i += 256) {
    const uint4 k0 = ks[i], v0 = vs[i];
    kd[i] = k0;
    vd[i] = v0;
  }
}

}  // namespace heatkv

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
  for (int i = threadIdx.x; i < total; i += 4 * 256) {
    uint4 kk[4], vv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = i + u * 256;
      if (j < total) {
        kk[u] = ks[j];
        vv[u] = vs[j];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = i + u * 256;
      if (j < total) {
        kd[j] = kk[u];
        vd[j] = vv[u];
      }
    }
  }
}

}  // namespace heatkv

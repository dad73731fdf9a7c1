// Cache update after a layer has run at scale k (Sec. 3.3): the layer's per-head
// runs are rewritten into the form the next scale reads.  Every block of rows to
// move was fixed by the planner (the schedule is static), so the kernel is a
// descriptor-driven streaming copy: 16 bytes per lane, a row of 256 bytes is one
// coalesced access of 16 lanes, K and V arenas handled by the same workgroup.
#include "device_util.h"
#include "kernels.h"

namespace heatkv {

namespace {

struct AppendParams {
  int chunks_per_row;  // row_bytes / 16
  int H, t_k;
  long long arena_tokens;
  const CopyDesc* descs;
  const uint4 *k_new, *v_new;
  uint4 *k_arena, *v_arena;
};

__global__ __launch_bounds__(256) void append_kernel(AppendParams p) {
  const CopyDesc d = p.descs[blockIdx.x];
  const int b = blockIdx.y;
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
    // up to four independent 16-byte loads in flight per lane and arena
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

}  // namespace

hipError_t launch_append(const AppendArgs& a, hipStream_t stream) {
  if (a.ndesc <= 0) return hipSuccess;
  if (a.row_bytes % 16 != 0) return hipErrorInvalidValue;
  AppendParams p{};
  p.chunks_per_row = a.row_bytes / 16;
  p.H = a.H;
  p.t_k = a.t_k;
  p.arena_tokens = a.arena_tokens;
  p.descs = a.descs;
  p.k_new = static_cast<const uint4*>(a.k_new);
  p.v_new = static_cast<const uint4*>(a.v_new);
  p.k_arena = static_cast<uint4*>(a.k_arena);
  p.v_arena = static_cast<uint4*>(a.v_arena);
  hipLaunchKernelGGL(append_kernel, dim3(a.ndesc, a.batch), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace heatkv

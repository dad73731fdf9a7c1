// Descriptor-driven row copy shared by the append kernel and by the attention kernels' fused append blocks.
#pragma once

#include "device_util.h"
#include "plan.h"

namespace heatkv {

struct CopyParams {
  int chunks_per_row;  // 16-byte chunks of a row of the new scale's tensors (row_bytes / 16)
  int kv_fp8;          // arena rows hold FP8 E4M3 codes: half the chunks per row, rows of the new scale are converted
  int H, t_k;
  long long arena_tokens;
  const CopyDesc* descs;
  const uint4 *k_new, *v_new;
  uint4 *k_arena, *v_arena;
};

// Four bf16 values (two 32-bit words, element 0 in the low half of w0) as four FP8 E4M3 codes, element 0 in the
// low byte: nearest-even (the conversion instruction's rounding), saturating at +-448 (the instruction itself
// turns larger magnitudes into NaN, so they are clamped first; a NaN fails the comparison and stays a NaN).
__device__ __forceinline__ unsigned bf16x4_to_e4m3(unsigned w0, unsigned w1) {
  auto sat = [](float x) { return fabsf(x) > 448.f ? copysignf(448.f, x) : x; };
  const float a = sat(__uint_as_float(w0 << 16)), b = sat(__uint_as_float(w0 & 0xffff0000u));
  const float c = sat(__uint_as_float(w1 << 16)), d = sat(__uint_as_float(w1 & 0xffff0000u));
  int p = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, p, true);
  return static_cast<unsigned>(p);
}
// 16 bf16 values (two 16-byte chunks) -> 16 codes (one chunk).
__device__ __forceinline__ uint4 bf16x16_to_e4m3(const uint4& lo, const uint4& hi) {
  return make_uint4(bf16x4_to_e4m3(lo.x, lo.y), bf16x4_to_e4m3(lo.z, lo.w), bf16x4_to_e4m3(hi.x, hi.y),
                    bf16x4_to_e4m3(hi.z, hi.w));
}

// One workgroup (256 lanes) moves descriptor `desc` of batch entry `b`: up to 128 contiguous rows, 16 bytes per
// lane, four independent loads in flight per lane and arena, K and V together.  Source and destination never
// overlap (the planner places the new region of a layer in free space).
__device__ __forceinline__ void copy_rows_block(const CopyParams& p, int desc, int b) {
  const CopyDesc d = p.descs[desc];
  const long long cpr = p.kv_fp8 ? p.chunks_per_row / 2 : p.chunks_per_row;  // chunks of an arena row
  const long long arena_base = static_cast<long long>(b) * p.arena_tokens * cpr;
  if (p.kv_fp8 && d.src_kind != 0) {  // rows of the new scale enter the 8-bit cache: one output chunk per lane and turn
    const long long s0 = (static_cast<long long>(b) * p.H * p.t_k + d.src_row) * p.chunks_per_row;
    const uint4 *ks = p.k_new + s0, *vs = p.v_new + s0;
    uint4* kd = p.k_arena + arena_base + static_cast<long long>(d.dst_row) * cpr;
    uint4* vd = p.v_arena + arena_base + static_cast<long long>(d.dst_row) * cpr;
    const int total = d.nrows * static_cast<int>(cpr);
    for (int i = threadIdx.x; i < total; i += 256) {
      const uint4 k0 = ks[2 * i], k1 = ks[2 * i + 1], v0 = vs[2 * i], v1 = vs[2 * i + 1];
      kd[i] = bf16x16_to_e4m3(k0, k1);
      vd[i] = bf16x16_to_e4m3(v0, v1);
    }
    return;
  }
  const long long dst0 = arena_base + static_cast<long long>(d.dst_row) * cpr;
  const uint4 *ks, *vs;
  if (d.src_kind == 0) {
    const long long s0 = arena_base + static_cast<long long>(d.src_row) * cpr;
    ks = p.k_arena + s0;
    vs = p.v_arena + s0;
  } else {
    const long long s0 = (static_cast<long long>(b) * p.H * p.t_k + d.src_row) * cpr;  // native rows: cpr both sides
    ks = p.k_new + s0;
    vs = p.v_new + s0;
  }
  uint4* kd = p.k_arena + dst0;
  uint4* vd = p.v_arena + dst0;
  const int total = d.nrows * static_cast<int>(cpr);
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

// Measurement aid: the bf16 matrix-core rate the chip sustains for given operand bits.  The attention and
// calibration kernels are priced against the datasheet peak; this loop of back-to-back, independent
// v_mfma_f32_32x32x16_bf16 instructions (no memory traffic, no vector ALU work) shows what the same matrix
// pipes deliver on the machine at hand, which depends on the operand data through the power-limited clock.
//
// This file is all of libheatkv_probe.so (C ABI in include/heatkv_probe.h); nothing here is linked into the
// product library.  It shares the LDS tile format of the product kernels (tile_lds.h), nothing else.
#include <string>
#include <type_traits>

#include <hip/hip_runtime_api.h>

#include "device_util.h"
#include "heatkv_probe.h"
#include "tile_lds.h"

namespace heatkv {

constexpr int kProbeOperands = 4096;  // 16-byte operand slots the kernel reads (64 KB)

__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint4* ops, float* out, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  union U {
    uint4 u;
    bf16x8 v;
  };
  U a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j].u = ops[(threadIdx.x * 16 + j) & (kProbeOperands - 1)];
    b[j].u = ops[(threadIdx.x * 16 + 8 + j) & (kProbeOperands - 1)];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + i) & 7].v, b[u].v, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// ---------------------------------------------------------------------------
// Tile-step model: the instruction mix, dependencies and memory traffic of one step of the bf16 attention
// kernel (per wavefront and 64-key tile: 16 score MFMAs fed from an LDS K tile, 32 scale FMAs, 32 exp2, 16
// packs, 16 pair sums, 16 PV MFMAs fed from an LDS V tile through transposing reads, a 32-value max chain,
// one barrier, and the HBM/L2 -> LDS copies of the next K and V tiles, in the kernel's hand-fixed issue order),
// without any of the kernel's bookkeeping: no ragged tiles, no masks, no rescaling, every workgroup streams the same 2 MB of tiles (they
// stay in L2).  Its throughput is what this mix sustains on the chip at hand; the numbers it computes mean
// nothing.  Two workgroups of four wavefronts per compute unit, as in the kernel.
// ---------------------------------------------------------------------------
constexpr int kRowBytes = tile::ROW_BYTES, kTileBytes = tile::BYTES, kModelTiles = 64;

__global__ __launch_bounds__(256, 2) void probe_tile_step_kernel(const char* kv, float* out, int iters) {
  __shared__ __attribute__((aligned(1024))) char lds[2][2][kTileBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 4 * kTileBytes / 4; i += 256)
    reinterpret_cast<unsigned*>(&lds[0][0][0])[i] = reinterpret_cast<const unsigned*>(kv)[i];
  __syncthreads();
  union U {
    uint4 u;
    bf16x8 v;
  };
  bf16x8 qreg[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    U t;
    t.u = reinterpret_cast<const uint4*>(kv)[(lane * 8 + i) & 1023];
    qreg[i] = t.v;
  }
  int k_off[8], v_off[4];
  tile::reader_off_k(lane, k_off);
  tile::reader_off_v(lane, v_off);
  const int ld_off_k = tile::loader_off_k(wave, lane);
  const int ld_off_v = tile::loader_off_v(wave, lane);
  const unsigned lds_base = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(
      reinterpret_cast<unsigned long long>((__attribute__((address_space(3))) char*)(&lds[0][0][0]))));
  // Copy of model tile `tile` (K: which = 0, V: which = 1) into buffer `buf`; all addresses stay inside the
  // 2 * kModelTiles tiles of `kv` and inside the 64 KB of LDS.
  auto issue = [&](int tile_i, int buf, int which) {
    const char* src = kv + (which * kModelTiles + (tile_i & (kModelTiles - 1))) * kTileBytes;
    tile::issue_full(lds_base + buf * (2 * kTileBytes) + which * kTileBytes, wave, which ? ld_off_v : ld_off_k, src);
  };
  f32x16 o[4], s_cur[2], s_nxt[2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s_cur[i][r] = static_cast<float>(qreg[i][r & 7]);
      s_nxt[i][r] = 0.f;
    }
  float l_run = 0.f, m_run = 0.f;
  const float c = 0.1f;
  const bf16x2 ones = {static_cast<bf16_t>(1.f), static_cast<bf16_t>(1.f)};
  union PB {
    bf16x8 v;
    bf16x2 h[4];
  };
  union VOperand {
    struct {
      s16x4 lo, hi;
    } s;
    bf16x8 v;
  };
  // One step in the attention kernel's hand-fixed issue order: 32 slots, one MFMA each followed by its share of
  // the vector and LDS work, scheduling fences between them.  Phases S(g) (the two K-steps of the score product that
  // go with 16-key chunk g, both 32-key blocks) and A(g) (P V of chunk g) alternate; the probabilities of chunk 0
  // are computed in the slots of S(0), those of chunk g+1 in the slots of A(g) and S(g+1), the maxima of the new
  // scores in the slots of A(3); every LDS operand is read a phase before its MFMA, the first ones right after
  // the barrier.
  auto step = [&](int it, auto buf_tag, f32x16 (&s_in)[2], f32x16 (&s_out)[2]) {
    constexpr int buf = decltype(buf_tag)::value;
    wait_vmcnt<0>();
    __syncthreads();
    const char* kt = lds[buf ^ 1][0];
    const char* vt = lds[buf][1];
    bf16x8 kop[8][2], vop[4][4];
    float e[4][8];
    PB pb[4];
    auto load_k = [&](int ks, int cb) {
      kop[ks][cb] = *reinterpret_cast<const bf16x8*>(kt + cb * 32 * kRowBytes + k_off[ks]);
    };
    auto load_v = [&](int chunk, int d) {
      const char* base = vt + 16 * chunk * kRowBytes + v_off[d];
      VOperand t;
      t.s.lo = lds_read_tr16(reinterpret_cast<const bf16_t*>(base));
      t.s.hi = lds_read_tr16(reinterpret_cast<const bf16_t*>(base + 8 * kRowBytes));
      vop[chunk][d] = t.v;
    };
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) load_k(i, cb);
#pragma unroll
    for (int d = 0; d < 4; ++d) load_v(0, d);
    issue(it + 2, buf, 0);
    issue(it + 1, buf ^ 1, 1);
    const float mc = m_run * c;
    auto p_half = [&](int chunk, int u) {
      const int cb = chunk >> 1, r = 8 * (chunk & 1) + u;
      e[chunk][u] = fast_exp2(fmaf(s_in[cb][r], c, -mc));
      if (u & 1) {
        pb[chunk].h[u >> 1] = bf16x2{static_cast<bf16_t>(e[chunk][u - 1]), static_cast<bf16_t>(e[chunk][u])};
        l_run = __builtin_amdgcn_fdot2_f32_bf16(pb[chunk].h[u >> 1], ones, l_run, false);
      }
    };
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_out[cb][r] = 0.f;
    fence();
    float mx = -INFINITY;
    auto s_slot = [&](int gch, int i, int& half) {
      const int ks = 2 * gch + (i >> 1), cb = i & 1;
      s_out[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[ks][cb], qreg[ks], s_out[cb], 0, 0, 0);
      fence();
      if (gch < 3) load_k(ks + 2, cb);
      const int n = gch == 0 ? 2 : 1;
      for (int u = 0; u < n; ++u) p_half(gch, half++);
      fence();
    };
    int half = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) s_slot(0, i, half);
#pragma unroll
    for (int gch = 0; gch < 4; ++gch) {
      half = 0;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[gch][d], pb[gch].v, o[d], 0, 0, 0);
        fence();
        if (gch < 3) {
          load_v(gch + 1, d);
          p_half(gch + 1, half++);
        } else {
#pragma unroll
          for (int r = 8 * d; r < 8 * d + 8; ++r) mx = fmaxf(mx, s_out[r >> 4][r & 15]);
          asm volatile("" : "+v"(mx));
        }
        fence();
      }
      if (gch < 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) s_slot(gch + 1, i, half);
      }
    }
    m_run = fmaxf(m_run, max_halves(mx) * 1e-6f);
  };
  for (int it = 0; it < iters; it += 2) {  // the two score sets swap roles from step to step
    step(it, std::integral_constant<int, 0>{}, s_cur, s_nxt);
    step(it + 1, std::integral_constant<int, 1>{}, s_nxt, s_cur);
  }
  wait_vmcnt<0>();
  float acc = l_run + m_run;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc += o[i][r];
  out[blockIdx.x * 256 + tid] = acc;
}

// Tile stream: the attention kernel's way of reading (HBM -> LDS copies of 1 KB per wavefront and instruction,
// two stages of a K and a V tile, a wait and a workgroup barrier per step, two workgroups per compute unit) with
// no arithmetic at all.  Workgroup w walks `steps` consecutive 32 KB steps of its own part of `src`; every thread
// folds one word of each landed step into a checksum, which is all it computes.
__global__ __launch_bounds__(256, 2) void probe_tile_stream_kernel(const char* src, int steps, unsigned* out) {
  __shared__ __attribute__((aligned(1024))) char lds[2][2 * kTileBytes];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const unsigned lds_base =
      static_cast<unsigned>(reinterpret_cast<unsigned long long>((__attribute__((address_space(3))) char*)(&lds[0][0])));
  const unsigned off = lane * 16;
  const char* base = src + static_cast<size_t>(blockIdx.x) * steps * (2 * kTileBytes);
  auto issue = [&](int t) {
    const char* s = base + static_cast<size_t>(t) * (2 * kTileBytes);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      tile::copy_1k(lds_base + (t & 1) * (2 * kTileBytes) + (4 * j + wave) * 1024, off, s + (4 * j + wave) * 1024);
  };
  issue(0);
  unsigned acc = 0;
  for (int t = 0; t < steps; ++t) {
    wait_vmcnt<0>();
    __syncthreads();
    if (t + 1 < steps) issue(t + 1);
    acc ^= *reinterpret_cast<const unsigned*>(&lds[t & 1][tid * 4]);
    // the stage read here is overwritten by the copy of step t + 2, which is issued after the next barrier
  }
  out[blockIdx.x * 256 + tid] = acc;
}

}  // namespace heatkv

namespace {

constexpr int kOk = 0, kEinval = -1, kEhip = -4;  // the HEATKV_* codes of heatkv.h
thread_local std::string g_probe_error;

int probe_fail(int code, const std::string& msg) {
  g_probe_error = msg;
  return code;
}
int probe_launch_result(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return probe_fail(kEhip, std::string(what) + ": " + hipGetErrorString(e));
  return kOk;
}

}  // namespace

extern "C" {

const char* heatkv_probe_last_error(void) { return g_probe_error.c_str(); }

size_t heatkv_probe_mfma_operand_bytes(void) { return size_t(heatkv::kProbeOperands) * 16; }

int heatkv_probe_mfma(const void* operands, float* out, int workgroups, int iters, void* stream) {
  if (!operands || !out) return probe_fail(kEinval, "null tensor pointer");
  if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20)) return probe_fail(kEinval, "probe size out of range");
  hipLaunchKernelGGL(heatkv::probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(operands), out, iters);
  return probe_launch_result("probe_mfma launch");
}

size_t heatkv_probe_tile_step_bytes(void) { return size_t(2) * heatkv::kModelTiles * heatkv::kTileBytes; }

int heatkv_probe_tile_step(const void* tiles, float* out, int workgroups, int iters, void* stream) {
  if (!tiles || !out) return probe_fail(kEinval, "null tensor pointer");
  if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || (iters & 1))
    return probe_fail(kEinval, "probe size out of range (iters must be even)");
  hipLaunchKernelGGL(heatkv::probe_tile_step_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(tiles), out, iters);
  return probe_launch_result("probe_tile_step launch");
}

size_t heatkv_probe_tile_stream_bytes(int workgroups, int steps) {
  if (workgroups <= 0 || workgroups > (1 << 20) || steps <= 0 || steps > (1 << 20)) return 0;
  return size_t(workgroups) * size_t(steps) * (2 * heatkv::kTileBytes);
}

int heatkv_probe_tile_stream(const void* src, size_t src_bytes, uint32_t* out, int workgroups, int steps, void* stream) {
  if (!src || !out) return probe_fail(kEinval, "null tensor pointer");
  const size_t need = heatkv_probe_tile_stream_bytes(workgroups, steps);
  if (need == 0) return probe_fail(kEinval, "probe size out of range");
  if (src_bytes < need) return probe_fail(kEinval, "probe source smaller than workgroups x steps x 32 KB");
  hipLaunchKernelGGL(heatkv::probe_tile_stream_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(src), steps, out);
  return probe_launch_result("probe_tile_stream launch");
}

}  // extern "C"

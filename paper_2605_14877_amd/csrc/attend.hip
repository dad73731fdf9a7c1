// Next-scale attention over the ragged per-head KV cache (Sec. 3.1 attention rows,
// Sec. 3.3 for which prior scales a head still holds).
//
// For head (b,h) the keys are the head's run of retained rows in the arena
// followed by the t_k rows of the current scale; queries are the t_k rows of
// the current scale.  Both kernels walk this virtual key sequence in tiles,
// keep running row maxima and row sums in fp32 (online softmax) and normalise
// once at the end.
#include <type_traits>

#include "device_util.h"
#include "kernels.h"

namespace heatkv {

namespace {

struct AttendParams {
  int H, batch, t_k;
  long long arena_tokens;
  const int32_t* run_row;
  const int32_t* run_len;
  const int32_t* head_order;
  const void *q, *k_cur, *v_cur, *k_arena, *v_arena;
  void* out;
  float sm_scale;
  int n_qtiles;
};

// ---------------------------------------------------------------------------
// bf16, d = 128: matrix-core kernel.
//
// Workgroup = 4 wavefronts, 128 queries (32 per wavefront); key tiles of 64
// rows are staged row-major in LDS.  Scores are produced transposed,
// S^T = K Q^T, with v_mfma_f32_32x32x16_bf16 so that one lane owns one query
// column: row maxima and sums are in-register reductions plus one exchange
// between the two wavefront halves, and the probabilities, rounded to bf16,
// already sit in the B-operand layout of the second product O^T += V^T P^T.
// V^T is read out of the row-major LDS tile with the transposing LDS read.
// ---------------------------------------------------------------------------
constexpr int BN = 64;     // keys per tile
constexpr int D128 = 128;
constexpr int KSTR = 136;  // LDS row stride of the K tile in elements (272 B: conflict-free 16-byte row reads)
constexpr int VSTR = 160;  // LDS row stride of the V tile in elements (320 B: best for the transposing read)

// NB = 32-query blocks per wavefront.  NB = 2 (256 queries per workgroup, one
// wavefront per SIMD, up to 512 registers) halves the LDS traffic per flop: every
// K or V operand fetched from LDS feeds two matrix instructions.  NB = 1 (128
// queries per workgroup, two wavefronts per SIMD) keeps more workgroups in
// flight for the short scales.
template <int NB>
__global__ __launch_bounds__(256, (NB == 1 ? 2 : 1)) void attend_bf16_d128_kernel(AttendParams p) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[BN * KSTR];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[BN * VSTR];
  constexpr int BM = 128 * NB;  // queries per workgroup

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, hl = lane >> 5;

  int id = blockIdx.x;
  const int qt = id % p.n_qtiles;
  id /= p.n_qtiles;
  const int b = id % p.batch;
  const int h = p.head_order[id / p.batch];

  const int t_k = p.t_k;
  const int n_prior = p.run_len[h];
  const int n_total = n_prior + t_k;
  const long long cur_off = (static_cast<long long>(b) * p.H + h) * t_k * D128;
  const long long run_off = (static_cast<long long>(b) * p.arena_tokens + p.run_row[h]) * D128;
  const bf16_t* k_prior = static_cast<const bf16_t*>(p.k_arena) + run_off;
  const bf16_t* v_prior = static_cast<const bf16_t*>(p.v_arena) + run_off;
  const bf16_t* k_cur = static_cast<const bf16_t*>(p.k_cur) + cur_off;
  const bf16_t* v_cur = static_cast<const bf16_t*>(p.v_cur) + cur_off;

  // Q as B operand: lane (n, hl) holds Q[row][16*ks + 8*hl .. +7] for ks = 0..7, for each of its NB rows.
  int q_row[NB];
  bf16x8 qreg[NB][8];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    q_row[nb] = qt * BM + wave * (32 * NB) + 32 * nb + n;
    const int ld = q_row[nb] < t_k ? q_row[nb] : t_k - 1;
    const bf16_t* qp = static_cast<const bf16_t*>(p.q) + cur_off + static_cast<long long>(ld) * D128 + 8 * hl;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[nb][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 o[NB][4];
  float m_run[NB], l_run[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m_run[nb] = -INFINITY;
    l_run[nb] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[nb][i][r] = 0.f;
  }
  const float c = p.sm_scale * kLog2e;

  const int n_tiles = (n_total + BN - 1) / BN;
  uint4 kbuf[4], vbuf[4];

  // Global -> register stage of the next tile.  Rows past the end of the key sequence re-read the last
  // valid row (finite data); their scores are masked to -inf in the last tile, so they contribute nothing.
  auto load_tile = [&](int tile) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = tid + 256 * i;
      const int row = chunk >> 4, col = chunk & 15;
      int g = tile * BN + row;
      g = g < n_total ? g : n_total - 1;
      const bool prior = g < n_prior;
      const long long off = static_cast<long long>(prior ? g : g - n_prior) * D128 + col * 8;
      kbuf[i] = ldg16((prior ? k_prior : k_cur) + off);
      vbuf[i] = ldg16((prior ? v_prior : v_cur) + off);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = tid + 256 * i;
      const int row = chunk >> 4, col = chunk & 15;
      *reinterpret_cast<uint4*>(&Ks[row * KSTR + col * 8]) = kbuf[i];
      *reinterpret_cast<uint4*>(&Vs[row * VSTR + col * 8]) = vbuf[i];
    }
  };

  // Address pattern of the transposing V read (see lds_read_tr16).
  const int tr_i = lane & 15, tr_grp = lane >> 4;
  const int tr_off = (4 * hl + (tr_i >> 2)) * VSTR + (tr_grp & 1) * 16 + 4 * (tr_i & 3);

  // The running reference m_run of a row is only raised when the tile maximum exceeds it by more than
  // kSlack in the exponent (base 2): probabilities are then at most 2^kSlack, far inside fp32/bf16 range,
  // the final division by the row sum makes the result independent of the reference, and the expensive
  // rescaling of the accumulators happens a handful of times per row instead of every few tiles.
  constexpr float kSlack = 8.f;
  const float slack_raw = kSlack / c;

  auto process_tile = [&](auto masked, int left) {
    // S^T = K Q^T for the 64 keys of the tile x this wavefront's 32*NB queries.
    f32x16 s[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[nb][cb][r] = 0.f;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(32 * cb + n) * KSTR + 16 * ks + 8 * hl]);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          s[nb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[nb][ks], s[nb][cb], 0, 0, 0);
      }
    // s[nb][cb][r] is key 32*cb + 8*(r/4) + 4*hl + r%4 of the tile, query block nb, column n.
    if constexpr (decltype(masked)::value) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (32 * cb + 8 * (r >> 2) + 4 * hl + (r & 3) >= left) s[nb][cb][r] = -INFINITY;
    }

    float mc[NB];
    bool raise = false;
    float mx[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float m = s[nb][0][0];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, s[nb][cb][r]);
      mx[nb] = max_halves(m);
      raise = raise || (mx[nb] > m_run[nb] + slack_raw);
    }
    if (__any(raise)) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const float m_new = fmaxf(m_run[nb], mx[nb]);
        const float alpha = fast_exp2((m_run[nb] - m_new) * c);
        m_run[nb] = m_new;
        l_run[nb] *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[nb][i][r] *= alpha;
      }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) mc[nb] = m_run[nb] * c;

    // P^T = 2^(S^T c - m c) in bf16, 16 keys at a time, each chunk feeding O^T += V^T P^T at once.
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 pb[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          float part = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float e = fast_exp2(fmaf(s[nb][cb][8 * ks + j], c, -mc[nb]));
            part += e;
            pb[nb][j] = static_cast<bf16_t>(e);
          }
          l_run[nb] += part;
        }
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk) {
          const bf16_t* base = &Vs[(32 * cb + 16 * ks) * VSTR + dblk * 32 + tr_off];
          union {
            struct {
              s16x4 lo, hi;
            } s;
            bf16x8 v;
          } a;
          a.s.lo = lds_read_tr16(base);
          a.s.hi = lds_read_tr16(base + 8 * VSTR);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            o[nb][dblk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pb[nb], o[nb][dblk], 0, 0, 0);
        }
      }
  };

  load_tile(0);
  for (int tile = 0; tile < n_tiles - 1; ++tile) {
    __syncthreads();
    store_tile();
    __syncthreads();
    load_tile(tile + 1);
    process_tile(std::false_type{}, BN);
  }
  __syncthreads();
  store_tile();
  __syncthreads();
  process_tile(std::true_type{}, n_total - (n_tiles - 1) * BN);

#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float l_tot = sum_halves(l_run[nb]);
    const float inv = 1.f / l_tot;
    if (q_row[nb] < t_k) {
      bf16_t* op = static_cast<bf16_t*>(p.out) + cur_off + static_cast<long long>(q_row[nb]) * D128;
#pragma unroll
      for (int dblk = 0; dblk < 4; ++dblk)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<bf16_t>(o[nb][dblk][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(op + dblk * 32 + 8 * g + 4 * hl) = v;
        }
    }
  }
}

// ---------------------------------------------------------------------------
// fp32 (any supported d): plain vector-ALU kernel, 16 queries per workgroup,
// 16 lanes per query, key tiles of 32 rows in LDS.
// ---------------------------------------------------------------------------
constexpr int FQ = 16;  // queries per workgroup
constexpr int FN = 32;  // keys per tile

template <int D>
__global__ __launch_bounds__(256) void attend_f32_kernel(AttendParams p) {
  __shared__ float Qs[FQ][D + 1];
  __shared__ float Ks[FN][D + 1];
  __shared__ float Vs[FN][D];
  __shared__ float Ps[FQ][FN];

  const int tid = threadIdx.x, r = tid >> 4, g = tid & 15;
  int id = blockIdx.x;
  const int qt = id % p.n_qtiles;
  id /= p.n_qtiles;
  const int b = id % p.batch;
  const int h = p.head_order[id / p.batch];

  const int t_k = p.t_k;
  const int n_prior = p.run_len[h];
  const int n_total = n_prior + t_k;
  const long long cur_off = (static_cast<long long>(b) * p.H + h) * t_k * D;
  const long long run_off = (static_cast<long long>(b) * p.arena_tokens + p.run_row[h]) * D;
  const float* k_prior = static_cast<const float*>(p.k_arena) + run_off;
  const float* v_prior = static_cast<const float*>(p.v_arena) + run_off;
  const float* k_cur = static_cast<const float*>(p.k_cur) + cur_off;
  const float* v_cur = static_cast<const float*>(p.v_cur) + cur_off;
  const float* q = static_cast<const float*>(p.q) + cur_off;

  for (int e = tid; e < FQ * D; e += 256) {
    const int rr = e / D, dd = e % D;
    const int row = qt * FQ + rr;
    Qs[rr][dd] = row < t_k ? q[static_cast<long long>(row) * D + dd] : 0.f;
  }

  constexpr int DPL = D / 16;  // output dims per lane
  float o[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) o[e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int n_tiles = (n_total + FN - 1) / FN;
  for (int tile = 0; tile < n_tiles; ++tile) {
    __syncthreads();
    for (int e = tid; e < FN * D; e += 256) {
      const int rr = e / D, dd = e % D;
      const int gk = tile * FN + rr;
      float kv = 0.f, vv = 0.f;
      if (gk < n_total) {
        const long long off = (gk < n_prior ? static_cast<long long>(gk) : static_cast<long long>(gk - n_prior)) * D + dd;
        kv = (gk < n_prior ? k_prior : k_cur)[off];
        vv = (gk < n_prior ? v_prior : v_cur)[off];
      }
      Ks[rr][dd] = kv;
      Vs[rr][dd] = vv;
    }
    __syncthreads();

    float s[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int j = g + 16 * jj;
      float acc = 0.f;
#pragma unroll 8
      for (int dd = 0; dd < D; ++dd) acc = fmaf(Qs[r][dd], Ks[j][dd], acc);
      s[jj] = tile * FN + j < n_total ? acc * p.sm_scale : -INFINITY;
    }
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 16));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = expf(m_run - m_new);
    const float p0 = expf(s[0] - m_new), p1 = expf(s[1] - m_new);
    float rowsum = p0 + p1;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) rowsum += __shfl_xor(rowsum, off, 16);
    l_run = l_run * alpha + rowsum;
    m_run = m_new;
    Ps[r][g] = p0;
    Ps[r][g + 16] = p1;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < DPL; ++e) {
      float acc = o[e] * alpha;
      for (int j = 0; j < FN; ++j) acc = fmaf(Ps[r][j], Vs[j][g + 16 * e], acc);
      o[e] = acc;
    }
  }

  const int row = qt * FQ + r;
  if (row < t_k) {
    float* op = static_cast<float*>(p.out) + cur_off + static_cast<long long>(row) * D;
    const float inv = 1.f / l_run;
#pragma unroll
    for (int e = 0; e < DPL; ++e) op[g + 16 * e] = o[e] * inv;
  }
}

}  // namespace

size_t attend_workspace_bytes(int, int, int, int, int, int) { return 0; }

hipError_t launch_attend(const AttendArgs& a, hipStream_t stream) {
  AttendParams p{};
  p.H = a.H;
  p.batch = a.batch;
  p.t_k = a.t_k;
  p.arena_tokens = a.arena_tokens;
  p.run_row = a.run_row;
  p.run_len = a.run_len;
  p.head_order = a.head_order;
  p.q = a.q;
  p.k_cur = a.k_cur;
  p.v_cur = a.v_cur;
  p.k_arena = a.k_arena;
  p.v_arena = a.v_arena;
  p.out = a.out;
  p.sm_scale = a.sm_scale;
  if (a.dtype == HEATKV_BF16) {
    if (a.d != 128) return hipErrorInvalidValue;
    // 256-query workgroups once they still fill the chip; 128-query workgroups for the short scales.
    const long long wide_groups = static_cast<long long>((a.t_k + 255) / 256) * a.H * a.batch;
    if (wide_groups >= 256) {
      p.n_qtiles = (a.t_k + 255) / 256;
      hipLaunchKernelGGL(attend_bf16_d128_kernel<2>, dim3(unsigned(wide_groups)), dim3(256), 0, stream, p);
    } else {
      p.n_qtiles = (a.t_k + 127) / 128;
      const unsigned grid = unsigned(p.n_qtiles) * a.H * a.batch;
      hipLaunchKernelGGL(attend_bf16_d128_kernel<1>, dim3(grid), dim3(256), 0, stream, p);
    }
  } else {
    p.n_qtiles = (a.t_k + FQ - 1) / FQ;
    const unsigned grid = unsigned(p.n_qtiles) * a.H * a.batch;
    if (a.d == 64)
      hipLaunchKernelGGL(attend_f32_kernel<64>, dim3(grid), dim3(256), 0, stream, p);
    else if (a.d == 128)
      hipLaunchKernelGGL(attend_f32_kernel<128>, dim3(grid), dim3(256), 0, stream, p);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace heatkv

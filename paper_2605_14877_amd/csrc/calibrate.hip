// Scale attention mass (Sec. 3.1, Eq. 2): for the queries of scale k1 over the
// uncompressed keys of scales 0..k1, the softmax mass that falls inside each
// key block k2, averaged over the query rows.
//
// The attention matrix is never materialised.  Key tiles never straddle two
// scale blocks; per query row the kernel keeps one running maximum and, for the
// block being walked, a sum of exponentials relative to that maximum.  At the
// end of a block the pair (sum, maximum at that moment) is parked in LDS; after
// the last block every parked sum is rescaled to the final maximum, which gives
// the row's normaliser and its per-block masses at once.  Row masses are then
// summed over the workgroup's rows in a fixed order and written as one partial
// per (head, query tile); a second kernel adds the partials in tile order, so
// the result is bit-reproducible (no floating-point atomics anywhere).
#include "device_util.h"
#include "kernels.h"

namespace heatkv {

namespace {

constexpr int MAXK = HEATKV_MAX_SCALES;

struct CalibParams {
  int H, batch, K, k1, t_k1, n_qtiles;
  int t[MAXK];
  int c[MAXK];  // c[k] = t[0] + .. + t[k]
  const void *q, *k_all;
  float sm_scale;
  float* partial;  // [batch*H][n_qtiles][K]
  float* mass;     // [batch*H][K]
};

// ---------------------------------------------------------------------------
// bf16, d = 128: S^T = K Q^T on the matrix cores, one lane per query column
// (same operand layout as the attention kernel), 128 queries per workgroup.
// ---------------------------------------------------------------------------
constexpr int CBM = 128;
constexpr int CBN = 64;
constexpr int CD = 128;
constexpr int CKSTR = 136;

__global__ __launch_bounds__(256, 2) void calibrate_bf16_d128_kernel(CalibParams p) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[CBN * CKSTR];
  __shared__ float blk_sum[MAXK][CBM];
  __shared__ float blk_max[MAXK][CBM];
  __shared__ float fin_max[CBM];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, hl = lane >> 5;
  int id = blockIdx.x;
  const int qt = id % p.n_qtiles;
  const int bh = id / p.n_qtiles;
  const int t_k1 = p.t_k1, k1 = p.k1;
  const int c_k1 = p.c[k1];

  const bf16_t* kbase = static_cast<const bf16_t*>(p.k_all) + static_cast<long long>(bh) * c_k1 * CD;
  const int q_row = qt * CBM + wave * 32 + n;
  const int q_row_ld = q_row < t_k1 ? q_row : t_k1 - 1;
  bf16x8 qreg[8];
  {
    const bf16_t* qp = static_cast<const bf16_t*>(p.q) + (static_cast<long long>(bh) * t_k1 + q_row_ld) * CD + 8 * hl;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }
  const float c = p.sm_scale * kLog2e;
  float m_run = -INFINITY;

  uint4 kbuf[4];
  auto load_tile = [&](int k2, int tile) {
    const int first = p.c[k2] - p.t[k2] + tile * CBN;
    const int left = p.t[k2] - tile * CBN;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int chunk = tid + 256 * i;
      const int row = chunk >> 4, col = chunk & 15;
      kbuf[i] = row < left ? ldg16(kbase + static_cast<long long>(first + row) * CD + col * 8) : make_uint4(0, 0, 0, 0);
    }
  };

  int k2 = 0, tile = 0;
  load_tile(0, 0);
  while (k2 <= k1) {
    float cur = 0.f;
    const int tiles_here = (p.t[k2] + CBN - 1) / CBN;
    for (; tile < tiles_here; ++tile) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int chunk = tid + 256 * i;
        *reinterpret_cast<uint4*>(&Ks[(chunk >> 4) * CKSTR + (chunk & 15) * 8]) = kbuf[i];
      }
      __syncthreads();
      if (tile + 1 < tiles_here)
        load_tile(k2, tile + 1);
      else if (k2 + 1 <= k1)
        load_tile(k2 + 1, 0);

      f32x16 s[2];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(32 * cb + n) * CKSTR + 16 * ks + 8 * hl]);
          s[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s[cb], 0, 0, 0);
        }
      }
      const int left = p.t[k2] - tile * CBN;
      if (left < CBN) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (32 * cb + 8 * (r >> 2) + 4 * hl + (r & 3) >= left) s[cb][r] = -INFINITY;
      }
      float mx = s[0][0];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[cb][r]);
      mx = fmaxf(mx, swap_halves(mx));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2((m_run - m_new) * c);
      const float mc = m_new * c;
      m_run = m_new;
      float rowsum = 0.f;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) rowsum += fast_exp2(fmaf(s[cb][r], c, -mc));
      cur = fmaf(cur, alpha, rowsum);
    }
    const float both = cur + swap_halves(cur);
    if (hl == 0) {
      blk_sum[k2][wave * 32 + n] = both;
      blk_max[k2][wave * 32 + n] = m_run;
    }
    ++k2;
    tile = 0;
  }
  if (hl == 0) fin_max[wave * 32 + n] = m_run;
  __syncthreads();

  // Row masses relative to the final maximum, normalised; rows past t_k1 contribute nothing.
  if (tid < CBM) {
    const float mf = fin_max[tid];
    float l = 0.f;
    for (int j = 0; j <= k1; ++j) {
      const float w = blk_sum[j][tid] * fast_exp2((blk_max[j][tid] - mf) * c);
      blk_sum[j][tid] = w;
      l += w;
    }
    const float inv = (qt * CBM + tid < t_k1) ? 1.f / l : 0.f;
    for (int j = 0; j <= k1; ++j) blk_sum[j][tid] *= inv;
  }
  __syncthreads();
  for (int j = wave; j <= k1; j += 4) {
    float v = blk_sum[j][lane] + blk_sum[j][lane + 64];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) p.partial[(static_cast<long long>(bh) * p.n_qtiles + qt) * p.K + j] = v;
  }
}

// ---------------------------------------------------------------------------
// fp32: vector-ALU kernel, 16 queries per workgroup, 16 lanes per query.
// ---------------------------------------------------------------------------
constexpr int FQ = 16;
constexpr int FN = 32;

template <int D>
__global__ __launch_bounds__(256) void calibrate_f32_kernel(CalibParams p) {
  __shared__ float Qs[FQ][D + 1];
  __shared__ float Ks[FN][D + 1];
  __shared__ float blk_sum[MAXK][FQ];
  __shared__ float blk_max[MAXK][FQ];

  const int tid = threadIdx.x, r = tid >> 4, g = tid & 15;
  int id = blockIdx.x;
  const int qt = id % p.n_qtiles;
  const int bh = id / p.n_qtiles;
  const int t_k1 = p.t_k1, k1 = p.k1;
  const float* kbase = static_cast<const float*>(p.k_all) + static_cast<long long>(bh) * p.c[k1] * D;
  const float* q = static_cast<const float*>(p.q) + static_cast<long long>(bh) * t_k1 * D;

  for (int e = tid; e < FQ * D; e += 256) {
    const int rr = e / D, dd = e % D;
    const int row = qt * FQ + rr;
    Qs[rr][dd] = row < t_k1 ? q[static_cast<long long>(row) * D + dd] : 0.f;
  }
  float m_run = -INFINITY;
  for (int k2 = 0; k2 <= k1; ++k2) {
    float cur = 0.f;
    const int first = p.c[k2] - p.t[k2];
    const int tiles_here = (p.t[k2] + FN - 1) / FN;
    for (int tile = 0; tile < tiles_here; ++tile) {
      const int left = p.t[k2] - tile * FN;
      __syncthreads();
      for (int e = tid; e < FN * D; e += 256) {
        const int rr = e / D, dd = e % D;
        Ks[rr][dd] = rr < left ? kbase[static_cast<long long>(first + tile * FN + rr) * D + dd] : 0.f;
      }
      __syncthreads();
      float s[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int j = g + 16 * jj;
        float acc = 0.f;
#pragma unroll 8
        for (int dd = 0; dd < D; ++dd) acc = fmaf(Qs[r][dd], Ks[j][dd], acc);
        s[jj] = j < left ? acc * p.sm_scale : -INFINITY;
      }
      float mx = fmaxf(s[0], s[1]);
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 16));
      const float m_new = fmaxf(m_run, mx);
      float rowsum = expf(s[0] - m_new) + expf(s[1] - m_new);
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) rowsum += __shfl_xor(rowsum, off, 16);
      cur = cur * expf(m_run - m_new) + rowsum;
      m_run = m_new;
    }
    if (g == 0) {
      blk_sum[k2][r] = cur;
      blk_max[k2][r] = m_run;
    }
  }
  __syncthreads();
  if (tid < FQ) {
    const float mf = blk_max[k1][tid];
    float l = 0.f;
    for (int j = 0; j <= k1; ++j) {
      const float w = blk_sum[j][tid] * expf(blk_max[j][tid] - mf);
      blk_sum[j][tid] = w;
      l += w;
    }
    const float inv = (qt * FQ + tid < t_k1) ? 1.f / l : 0.f;
    for (int j = 0; j <= k1; ++j) blk_sum[j][tid] *= inv;
  }
  __syncthreads();
  if (tid <= k1) {
    float v = 0.f;
    for (int rr = 0; rr < FQ; ++rr) v += blk_sum[tid][rr];
    p.partial[(static_cast<long long>(bh) * p.n_qtiles + qt) * p.K + tid] = v;
  }
}

// Adds the per-tile partial sums in tile order and divides by the number of query rows.
__global__ void calibrate_finish_kernel(CalibParams p) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = p.batch * p.H * p.K;
  if (i >= total) return;
  const int j = i % p.K;
  const long long bh = i / p.K;
  float v = 0.f;
  if (j <= p.k1) {
    for (int qt = 0; qt < p.n_qtiles; ++qt) v += p.partial[(bh * p.n_qtiles + qt) * p.K + j];
    v /= static_cast<float>(p.t_k1);
  }
  p.mass[i] = v;
}

__global__ void accumulate_beta_kernel(int H, int batch, int K, int layer, int k1, const float* mass, float weight,
                                       float* beta) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= H * K) return;
  const int h = i / K, k2 = i % K;
  float v = 0.f;
  for (int b = 0; b < batch; ++b) v += mass[(static_cast<long long>(b) * H + h) * K + k2];
  beta[((static_cast<long long>(layer) * H + h) * K + k1) * K + k2] += weight * v;
}

int queries_per_tile(int dtype) { return dtype == HEATKV_BF16 ? CBM : FQ; }

}  // namespace

size_t calibrate_workspace_bytes(int dtype, int, int H, int batch, int K, int t_k1) {
  const int qpt = queries_per_tile(dtype);
  const size_t n_qtiles = size_t((t_k1 + qpt - 1) / qpt);
  return size_t(batch) * H * n_qtiles * K * sizeof(float);
}

hipError_t launch_calibrate(const CalibrateArgs& a, hipStream_t stream) {
  CalibParams p{};
  p.H = a.H;
  p.batch = a.batch;
  p.K = a.K;
  p.k1 = a.k1;
  p.t_k1 = a.t[a.k1];
  int acc = 0;
  for (int k = 0; k < a.K; ++k) {
    p.t[k] = a.t[k];
    acc += a.t[k];
    p.c[k] = acc;
  }
  const int qpt = queries_per_tile(a.dtype);
  p.n_qtiles = (p.t_k1 + qpt - 1) / qpt;
  p.q = a.q;
  p.k_all = a.k_all;
  p.sm_scale = a.sm_scale;
  p.partial = static_cast<float*>(a.ws);
  p.mass = a.mass;
  const unsigned grid = unsigned(p.n_qtiles) * a.H * a.batch;
  if (a.dtype == HEATKV_BF16) {
    if (a.d != 128) return hipErrorInvalidValue;
    hipLaunchKernelGGL(calibrate_bf16_d128_kernel, dim3(grid), dim3(256), 0, stream, p);
  } else if (a.d == 64) {
    hipLaunchKernelGGL(calibrate_f32_kernel<64>, dim3(grid), dim3(256), 0, stream, p);
  } else if (a.d == 128) {
    hipLaunchKernelGGL(calibrate_f32_kernel<128>, dim3(grid), dim3(256), 0, stream, p);
  } else {
    return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int total = a.batch * a.H * a.K;
  hipLaunchKernelGGL(calibrate_finish_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_accumulate_beta(int H, int batch, int K, int layer, int k1, const float* mass, float weight,
                                  float* beta, hipStream_t stream) {
  const int total = H * K;
  hipLaunchKernelGGL(accumulate_beta_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, H, batch, K, layer, k1,
                     mass, weight, beta);
  return hipGetLastError();
}

}  // namespace heatkv

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
// summed over 128 rows at a time in a fixed order and written as one partial per
// (head, 128 query rows); a second kernel adds the partials in row order, so the
// result is bit-reproducible (no floating-point atomics anywhere).
#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>

#include "device_util.h"
#include "kernels.h"
#include "tile_lds.h"

namespace heatkv {

namespace {

constexpr int MAXK = HEATKV_MAX_SCALES;

// One query scale of a launch.  A launch may cover several (calibration data of all scales is available at
// once, unlike generation); their workgroups are laid out one scale after the other, largest scale first.
struct ScaleJob {
  int k1;
  int block_begin;  // first workgroup id of this scale (a multiple of 8 in the bf16 kernel)
  const void *q, *k_all;
  float* partial;  // [batch*H][n_qtiles][K]
  float* mass;     // [batch*H][K], may be null in the accumulating variant
};

struct CalibParams {
  int H, batch, K, n_scales;
  int t[MAXK];
  int c[MAXK];  // c[k] = t[0] + .. + t[k]
  ScaleJob job[MAXK];
  float sm_scale;
  float* beta;  // [L][H][K][K] or null
  float weight;
  int layer;
};

// The scale a workgroup belongs to (workgroup-uniform, a handful of scalar compares).
__device__ __forceinline__ int scale_of_block(const CalibParams& p, int block) {
  int si = 0;
  while (si + 1 < p.n_scales && block >= p.job[si + 1].block_begin) ++si;
  return si;
}

// ---------------------------------------------------------------------------
// bf16, d = 128 or 64: S^T = K Q^T on the matrix cores, one lane per query column
// (same operand layout, LDS tile format and HBM -> LDS copy as the attention
// kernel).  Two instances.  CSETS = 1: 128 queries per workgroup, one set of 32 per
// wavefront, three workgroups per compute unit.  CSETS = 2: 256 queries per
// workgroup; every wavefront owns two sets of 32 (rows w*32 + n and 128 + w*32 + n
// of the tile) and runs both against each K operand it has read from LDS, so a K
// tile is copied and read once per 256 queries and the matrix-core work of one set
// overlaps the exponentials of the other inside the wavefront; two workgroups per
// compute unit.  On a full chip the two are equally fast (two wavefronts per SIMD
// with twice the independent work against three); the launcher takes the second
// when its workgroups fill their 512 slots at least once, which then needs fewer,
// longer workgroups and ends with a shorter tail.
// ---------------------------------------------------------------------------
constexpr int CBM1 = 128;  // queries per set of four wavefronts
constexpr int CBN = tile::ROWS;

// Dynamic LDS: two K tiles, then blk_sum[k1+1][rows], blk_max[k1+1][rows], fin_max[rows] (floats), rows = the
// queries of a workgroup.
__host__ __device__ constexpr size_t calib_lds_bytes(int k1, int csets, int d) {
  return 2 * size_t(CBN * 2 * d) + (2 * size_t(k1 + 1) + 1) * (CBM1 * csets) * sizeof(float);
}

template <int CSETS, int CD>
__global__ __launch_bounds__(256, CSETS == 1 ? 3 : 2) void calibrate_bf16_kernel(CalibParams p) {
  static_assert(CD == 128 || CD == 64, "head dimension 128 or 64");
  constexpr int CROW_BYTES = 2 * CD;            // one bf16 row
  constexpr int CTILE_BYTES = CBN * CROW_BYTES;  // 16 KB or 8 KB
  constexpr int NK = CD / 16;                    // MFMA steps of a score block
  constexpr int CBM = CBM1 * CSETS;  // queries per workgroup
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const ScaleJob& job = p.job[scale_of_block(p, blockIdx.x)];
  const int k1 = job.k1, t_k1 = p.t[k1];
  const int n_qtiles = (t_k1 + CBM - 1) / CBM;
  const int block = blockIdx.x - job.block_begin;
  float* blk_sum = reinterpret_cast<float*>(lds + 2 * CTILE_BYTES);
  float* blk_max = blk_sum + (k1 + 1) * CBM;
  float* fin_max = blk_max + (k1 + 1) * CBM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hl = lane >> 5;

  // All query tiles of one (batch row, head) read the same keys: give them ids on one XCD (id % 8).
  const int xcd = block & 7, slot = block >> 3;  // block_begin is a multiple of 8: block & 7 is the hardware XCD
  const int bh = (slot / n_qtiles) * 8 + xcd;
  if (bh >= p.batch * p.H) return;
  const int qt = slot % n_qtiles;
  const int c_k1 = p.c[k1];

  const char* kbase = reinterpret_cast<const char*>(static_cast<const bf16_t*>(job.k_all) +
                                                    static_cast<long long>(bh) * c_k1 * CD);
  // The second set of a tile exists only if the tile reaches past its first 128 rows (workgroup-uniform).
  const bool two_sets = CSETS == 2 && qt * CBM + 128 < t_k1;
  bf16x8 qreg[CSETS][NK];
#pragma unroll
  for (int qs = 0; qs < CSETS; ++qs) {
    const int q_row = qt * CBM + qs * 128 + wave * 32 + n;
    const int ld = q_row < t_k1 ? q_row : t_k1 - 1;
    const bf16_t* qp = static_cast<const bf16_t*>(job.q) + (static_cast<long long>(bh) * t_k1 + ld) * CD + 8 * hl;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) qreg[qs][ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }
  const float c = p.sm_scale * kLog2e;

  // HBM -> LDS copy of one K tile in the tile format shared with the attention kernel (tile_lds.h: raw
  // global_load_lds, explicit ordering by s_waitcnt vmcnt + barrier).
  const int ld_off = tile::loader_off_k<CROW_BYTES>(wave, lane);
  const unsigned lds_base =
      static_cast<unsigned>(reinterpret_cast<unsigned long long>((__attribute__((address_space(3))) char*)(&lds[0])));
  auto issue_tile = [&](int k2, int tile_i, int buf) {
    const int left = p.t[k2] - tile_i * CBN;
    const char* kb = kbase + static_cast<long long>(p.c[k2] - p.t[k2] + tile_i * CBN) * CROW_BYTES;
    const unsigned kd = lds_base + buf * CTILE_BYTES;
    if (left >= CBN)
      tile::issue_full<CROW_BYTES>(kd, wave, ld_off, kb);
    else  // ragged tile: rows past the end re-read the last valid row
      tile::issue_ragged<false, CROW_BYTES>(kd, wave, lane, left, kb);
  };
  int k_off[NK];
  tile::reader_off_k<CROW_BYTES>(lane, k_off);

  float m_run[CSETS], cur[CSETS];
#pragma unroll
  for (int qs = 0; qs < CSETS; ++qs) {
    m_run[qs] = -INFINITY;
    cur[qs] = 0.f;
  }
  int k2 = 0, tile = 0;  // the tile being computed

  auto tile_step = [&](auto buf_tag) {
    constexpr int buf = decltype(buf_tag)::value;
    // successor of (k2, tile) in block-major order
    const int tiles_here = (p.t[k2] + CBN - 1) / CBN;
    const bool last_of_block = tile + 1 >= tiles_here;
    const int nk2 = last_of_block ? k2 + 1 : k2, ntile = last_of_block ? 0 : tile + 1;
    wait_vmcnt<0>();
    __syncthreads();
    if (nk2 <= k1) issue_tile(nk2, ntile, buf ^ 1);
    const char* kt = lds + buf * CTILE_BYTES;

    bf16x8 ka[2][NK];
#pragma unroll
    for (int ks = 0; ks < NK; ++ks)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
        ka[cb][ks] = *reinterpret_cast<const bf16x8*>(kt + cb * 32 * CROW_BYTES + k_off[ks]);
    const int left = p.t[k2] - tile * CBN;
#pragma unroll
    for (int qs = 0; qs < CSETS; ++qs) {
      if (qs == 1 && !two_sets) break;
      f32x16 s[2];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NK; ++ks)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
          s[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[cb][ks], qreg[qs][ks], s[cb], 0, 0, 0);
      if (qs == 0) {  // all sixteen operand reads go out before the first MFMA instead of two at a time
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * NK, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NK, 0);
      }

      if (left < CBN) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (32 * cb + 8 * (r >> 2) + 4 * hl + (r & 3) >= left) s[cb][r] = -INFINITY;
      }
      // Probabilities are taken relative to the running reference m_run, which is only brought up to the true
      // row maximum when it has fallen too far behind: as long as no score exceeds it by more than 8 in the
      // base-2 exponent a lane's 32 probabilities of the tile sum to at most 2^13, so a larger sum, an infinity
      // or a NaN (the first tile, where m_run is still -inf) sends the whole wavefront through the exact path,
      // which finds the tile maximum, rescales what the block has summed so far and redoes the tile's
      // exponentials.  The masses are ratios of such sums, so they do not depend on the reference; the max
      // chain, one vector instruction per two scores, leaves the common path.
      float mc = m_run[qs] * c;
      float rs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) rs[r & 3] += fast_exp2(fmaf(s[cb][r], c, -mc));
      float tile_sum = (rs[0] + rs[1]) + (rs[2] + rs[3]);
      if (__any(!(tile_sum <= 8192.f))) {
        float mx = s[0][0];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[cb][r]);
        mx = max_halves(mx);
        const float m_new = fmaxf(m_run[qs], mx);
        cur[qs] *= fast_exp2((m_run[qs] - m_new) * c);
        m_run[qs] = m_new;
        mc = m_new * c;
#pragma unroll
        for (int i = 0; i < 4; ++i) rs[i] = 0.f;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r) rs[r & 3] += fast_exp2(fmaf(s[cb][r], c, -mc));
        tile_sum = (rs[0] + rs[1]) + (rs[2] + rs[3]);
      }
      cur[qs] += tile_sum;

      if (last_of_block) {
        const float both = sum_halves(cur[qs]);
        if (hl == 0) {
          blk_sum[k2 * CBM + qs * 128 + wave * 32 + n] = both;
          blk_max[k2 * CBM + qs * 128 + wave * 32 + n] = m_run[qs];
        }
        cur[qs] = 0.f;
      }
    }
    k2 = nk2;
    tile = ntile;
  };

  issue_tile(0, 0, 0);
  while (true) {
    tile_step(std::integral_constant<int, 0>{});
    if (k2 > k1) break;
    tile_step(std::integral_constant<int, 1>{});
    if (k2 > k1) break;
  }
  if (hl == 0) {
#pragma unroll
    for (int qs = 0; qs < CSETS; ++qs) fin_max[qs * 128 + wave * 32 + n] = m_run[qs];
  }
  __syncthreads();

  // Row masses relative to the final maximum, normalised; rows past t_k1 contribute nothing.
  if (tid < 128 || two_sets) {  // one thread per query row of the tile; rows of an absent second set hold nothing
    const float mf = fin_max[tid];
    float l = 0.f;
    for (int j = 0; j <= k1; ++j) {
      const float w = blk_sum[j * CBM + tid] * fast_exp2((blk_max[j * CBM + tid] - mf) * c);
      blk_sum[j * CBM + tid] = w;
      l += w;
    }
    const float inv = (qt * CBM + tid < t_k1) ? 1.f / l : 0.f;
    for (int j = 0; j <= k1; ++j) blk_sum[j * CBM + tid] *= inv;
  }
  __syncthreads();
  // One partial per 128 query rows whichever the instance: a set of the two-set instance holds exactly the rows of
  // one query tile of the other and sums them in the same order, so both write the same bits to the same places.
  const int n_parts = (t_k1 + CBM1 - 1) / CBM1;
  for (int j = wave; j <= k1; j += 4) {
#pragma unroll
    for (int qs = 0; qs < CSETS; ++qs) {
      if (qs == 1 && !two_sets) break;
      float v = blk_sum[j * CBM + qs * CBM1 + lane] + blk_sum[j * CBM + qs * CBM1 + lane + 64];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0) job.partial[(static_cast<long long>(bh) * n_parts + CSETS * qt + qs) * p.K + j] = v;
    }
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
  const ScaleJob& job = p.job[scale_of_block(p, blockIdx.x)];
  const int k1 = job.k1, t_k1 = p.t[k1];
  const int n_qtiles = (t_k1 + FQ - 1) / FQ;
  const int id = blockIdx.x - job.block_begin;
  const int qt = id % n_qtiles;
  const int bh = id / n_qtiles;
  const float* kbase = static_cast<const float*>(job.k_all) + static_cast<long long>(bh) * p.c[k1] * D;
  const float* q = static_cast<const float*>(job.q) + static_cast<long long>(bh) * t_k1 * D;

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
    job.partial[(static_cast<long long>(bh) * n_qtiles + qt) * p.K + tid] = v;
  }
}

// Sum of one (batch row, head, key block) entry over the query tiles, in tile order, divided by the number of
// query rows.  The loads of a group of eight go out together (the kernel is a chain of dependent additions fed
// by L2 latency otherwise); the additions keep the order.
__device__ __forceinline__ float tile_sum_in_order(const CalibParams& p, const ScaleJob& job, int n_qtiles,
                                                   long long bh, int j) {
  if (j > job.k1) return 0.f;
  const float* src = job.partial + bh * n_qtiles * p.K + j;
  float v = 0.f;
  int qt = 0;
  for (; qt + 8 <= n_qtiles; qt += 8) {
    float x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = src[static_cast<long long>(qt + u) * p.K];
#pragma unroll
    for (int u = 0; u < 8; ++u) v += x[u];
  }
  for (; qt < n_qtiles; ++qt) v += src[static_cast<long long>(qt) * p.K];
  return v / static_cast<float>(p.t[job.k1]);
}

// Adds the per-tile partial sums in tile order and divides by the number of query rows.  blockIdx.y = scale of
// the launch; qpt = query rows per tile of the kernel that wrote the partials.
__global__ void calibrate_finish_kernel(CalibParams p, int qpt) {
  const ScaleJob& job = p.job[blockIdx.y];
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = p.batch * p.H * p.K;
  if (i >= total) return;
  job.mass[i] = tile_sum_in_order(p, job, (p.t[job.k1] + qpt - 1) / qpt, i / p.K, i % p.K);
}

// Same reduction followed by the dataset average in one pass: one thread per (head, key block) walks the batch
// rows in order, so the result has the bits of calibrate_finish_kernel followed by accumulate_beta_kernel.
__global__ void calibrate_finish_accumulate_kernel(CalibParams p, int qpt) {
  const ScaleJob& job = p.job[blockIdx.y];
  const int n_qtiles = (p.t[job.k1] + qpt - 1) / qpt;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= p.H * p.K) return;
  const int h = i / p.K, j = i % p.K;
  float acc = 0.f;
  for (int b = 0; b < p.batch; ++b) {
    const long long bh = static_cast<long long>(b) * p.H + h;
    const float v = tile_sum_in_order(p, job, n_qtiles, bh, j);
    if (job.mass) job.mass[bh * p.K + j] = v;
    acc += v;
  }
  p.beta[((static_cast<long long>(p.layer) * p.H + h) * p.K + job.k1) * p.K + j] += p.weight * acc;
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

// Query rows per partial sum.
int queries_per_tile(int dtype) { return dtype == HEATKV_BF16 ? CBM1 : FQ; }

}  // namespace

size_t calibrate_workspace_bytes(int dtype, int, int H, int batch, int K, int t_k1) {
  const int qpt = queries_per_tile(dtype);
  const size_t n_qtiles = size_t((t_k1 + qpt - 1) / qpt);
  return size_t(batch) * H * n_qtiles * K * sizeof(float);
}

// Several scales in one launch: each scale's partials start on a 256-byte boundary.
size_t calibrate_scales_workspace_bytes(int dtype, int d, int H, int batch, int K, const int32_t* t, int n_scales,
                                        const int32_t* k1) {
  size_t total = 0;
  for (int i = 0; i < n_scales; ++i)
    total += (calibrate_workspace_bytes(dtype, d, H, batch, K, t[k1[i]]) + 255) / 256 * 256;
  return total;
}

hipError_t launch_calibrate(const CalibrateArgs& a, hipStream_t stream) {
  if (a.n_scales < 1 || a.n_scales > MAXK) return hipErrorInvalidValue;
  CalibParams p{};
  p.H = a.H;
  p.batch = a.batch;
  p.K = a.K;
  p.n_scales = a.n_scales;
  int acc = 0;
  for (int k = 0; k < a.K; ++k) {
    p.t[k] = a.t[k];
    acc += a.t[k];
    p.c[k] = acc;
  }
  p.sm_scale = a.sm_scale;
  p.beta = a.beta;
  p.weight = a.weight;
  p.layer = a.layer;
  const bool mfma = a.dtype == HEATKV_BF16;
  // bf16: the instance with two query sets per wavefront if its workgroups fill their 512 slots at least once.
  // Both leave one partial per 128 query rows (qpt), bit for bit the same ones.
  const int qpt = queries_per_tile(a.dtype);
  int rows_per_block = qpt;
  if (mfma) {
    unsigned long long wide_blocks = 0;
    for (int i = 0; i < a.n_scales; ++i)
      wide_blocks += (unsigned long long)((a.t[a.k1[i]] + 2 * CBM1 - 1) / (2 * CBM1)) * a.H * a.batch;
    if (wide_blocks >= 512) rows_per_block = 2 * CBM1;
  }
  if (mfma && a.d != 128 && a.d != 64) return hipErrorInvalidValue;
  if (!mfma && a.d != 64 && a.d != 128) return hipErrorInvalidValue;
  // Largest scale first: its workgroups are the long ones, the short ones then fill the gaps they leave.
  int order[MAXK];
  for (int i = 0; i < a.n_scales; ++i) order[i] = i;
  std::stable_sort(order, order + a.n_scales, [&](int x, int y) { return a.t[a.k1[x]] > a.t[a.k1[y]]; });
  // In the bf16 kernel the (batch row, head) pairs are padded to a multiple of 8 so that id % 8 is the XCD.
  const unsigned pairs = mfma ? (unsigned(a.H) * a.batch + 7) / 8 * 8 : unsigned(a.H) * a.batch;
  unsigned blocks = 0;
  size_t ws_off = 0;
  int k1_max = 0;
  for (int i = 0; i < a.n_scales; ++i) {
    const int src = order[i];
    ScaleJob& job = p.job[i];
    job.k1 = a.k1[src];
    job.block_begin = int(blocks);
    job.q = a.q[src];
    job.k_all = a.k_all[src];
    job.partial = reinterpret_cast<float*>(static_cast<char*>(a.ws) + ws_off);
    job.mass = a.mass[src];
    blocks += unsigned((a.t[job.k1] + rows_per_block - 1) / rows_per_block) * pairs;
    ws_off += (calibrate_workspace_bytes(a.dtype, a.d, a.H, a.batch, a.K, a.t[job.k1]) + 255) / 256 * 256;
    k1_max = job.k1 > k1_max ? job.k1 : k1_max;
  }
  if (mfma) {
    // Many scales need more than the default 64 KB of dynamic LDS for the parked block sums: raise the limit to
    // what the largest scale count can ask for, once per device.
    static std::atomic<unsigned long long> raised{0};  // one bit per device ordinal below 64
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !(raised.load(std::memory_order_acquire) >> dev & 1)) {
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&calibrate_bf16_kernel<2, 128>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, int(calib_lds_bytes(MAXK - 1, 2, 128)));
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&calibrate_bf16_kernel<2, 64>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, int(calib_lds_bytes(MAXK - 1, 2, 64)));
      if (e != hipSuccess) return e;
      if (dev >= 0 && dev < 64) raised.fetch_or(1ull << dev, std::memory_order_release);
    }
    const size_t lds_bytes = calib_lds_bytes(k1_max, rows_per_block == CBM1 ? 1 : 2, a.d);
    if (a.d == 128 && rows_per_block == CBM1)
      hipLaunchKernelGGL((calibrate_bf16_kernel<1, 128>), dim3(blocks), dim3(256), lds_bytes, stream, p);
    else if (a.d == 128)
      hipLaunchKernelGGL((calibrate_bf16_kernel<2, 128>), dim3(blocks), dim3(256), lds_bytes, stream, p);
    else if (rows_per_block == CBM1)
      hipLaunchKernelGGL((calibrate_bf16_kernel<1, 64>), dim3(blocks), dim3(256), lds_bytes, stream, p);
    else
      hipLaunchKernelGGL((calibrate_bf16_kernel<2, 64>), dim3(blocks), dim3(256), lds_bytes, stream, p);
  }
  else if (a.d == 64)
    hipLaunchKernelGGL(calibrate_f32_kernel<64>, dim3(blocks), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(calibrate_f32_kernel<128>, dim3(blocks), dim3(256), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.beta) {
    hipLaunchKernelGGL(calibrate_finish_accumulate_kernel, dim3((a.H * a.K + 255) / 256, a.n_scales), dim3(256), 0,
                       stream, p, qpt);
  } else {
    const int total = a.batch * a.H * a.K;
    hipLaunchKernelGGL(calibrate_finish_kernel, dim3((total + 255) / 256, a.n_scales), dim3(256), 0, stream, p, qpt);
  }
  return hipGetLastError();
}

// Workspace for callers that cannot allocate: the per-tile partial sums live in this file-scope device array
// instead of a caller buffer.  Every GPU the library runs on holds its own copy at its own address until the
// process ends; the array's name is only a host-side handle, the device address comes from
// hipGetSymbolAddress, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[kCalibrateStaticBytes];

hipError_t calibrate_static_workspace(void** ptr) {
  static std::mutex mu;
  static void* per_device[64] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  return hipSuccess;
}

hipError_t launch_accumulate_beta(int H, int batch, int K, int layer, int k1, const float* mass, float weight,
                                  float* beta, hipStream_t stream) {
  const int total = H * K;
  hipLaunchKernelGGL(accumulate_beta_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, H, batch, K, layer, k1,
                     mass, weight, beta);
  return hipGetLastError();
}

}  // namespace heatkv

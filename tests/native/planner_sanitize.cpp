// Host-only driver for the planner, built with AddressSanitizer and UBSan by tests/test_planner_sanitizers.py.
// It builds schedules for seeded random beta tables over several shapes and variants and replays the accessors
// that walk the plan's tables; any out-of-bounds access or undefined behaviour aborts the run.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "plan.h"

static unsigned long long g_state = 88172645463325252ull;
static double rnd() {
  g_state ^= g_state << 13;
  g_state ^= g_state >> 7;
  g_state ^= g_state << 17;
  return double(g_state % 1000003) / 1000003.0;
}

static int run_case(int L, int H, const std::vector<int32_t>& t, int sinks, int variant, int factor) {
  const int K = int(t.size());
  heatkv_shape shape{L, H, 128, K, 2, HEATKV_BF16, t.data()};
  heatkv_plan p;
  if (heatkv::init_shape(&p, &shape)) return 1;
  p.sinks = sinks;
  p.variant = variant;
  p.from_schedule = true;
  long long prior = 0;
  for (int k = 0; k + 1 < K; ++k) prior += t[k];
  p.B = (long long)L * H * prior / factor;
  std::vector<float> beta(size_t(L) * H * K * K, 0.f);
  for (size_t head = 0; head < size_t(L) * H; ++head)
    for (int k1 = 0; k1 < K; ++k1) {
      double sum = 0;
      for (int k2 = 0; k2 <= k1; ++k2) sum += (beta[(head * K + k1) * K + k2] = float(rnd() + 1e-3));
      for (int k2 = 0; k2 <= k1; ++k2) beta[(head * K + k1) * K + k2] /= float(sum);
    }
  {  // the rank diagnostics walk the same table: three "runs" made of shifted copies of it
    std::vector<float> runs(3 * beta.size());
    for (int r = 0; r < 3; ++r)
      for (size_t i = 0; i < beta.size(); ++i) runs[r * beta.size() + i] = beta[(i + r * 7) % beta.size()];
    std::vector<double> sc(size_t(K) * L * H), disp(K);
    if (sinks <= K - 2) {
      if (heatkv::rank_scores(&shape, beta.data(), sinks, variant, sc.data())) return 8;
      if (heatkv::rank_dispersion(&shape, runs.data(), 3, sinks, variant, disp.data())) return 9;
    }
  }
  int rc = heatkv::build_sets(&p, beta.data());
  if (rc == HEATKV_EBUDGET) return 0;  // legitimate outcome for tight budgets
  if (rc) return 2;
  if (heatkv::derive_layout(&p)) return 3;
  // walk everything the kernels would read
  long long checksum = 0;
  for (int k = 0; k < K; ++k)
    for (int l = 0; l < L; ++l) {
      for (int h = 0; h < H; ++h) {
        const int32_t row = p.run_row[p.idx(k, l, h)], len = p.run_len[p.idx(k, l, h)];
        if (row < 0 || row + len > p.arena_tokens) return 4;
        checksum += row + len + p.head_order[p.idx(k, l, h)];
      }
      const long long b = p.desc_begin[p.idx(k, l)];
      for (int i = 0; i < p.desc_count[p.idx(k, l)]; ++i) {
        const heatkv::CopyDesc& d = p.descs[size_t(b + i)];
        if (d.nrows <= 0 || d.dst_row < 0 || d.dst_row + d.nrows > p.arena_tokens) return 5;
        if (d.src_kind == 0 && (d.src_row < 0 || d.src_row + d.nrows > p.arena_tokens)) return 6;
        if (d.src_kind == 1 && (d.src_row < 0 || d.src_row + d.nrows > H * t[k])) return 7;
        checksum += d.nrows;
      }
    }
  std::printf("L=%d H=%d K=%d s=%d variant=%d 1/%d: arena %lld rows, budget %lld, checksum %lld\n", L, H, K, sinks,
              variant, factor, (long long)p.arena_tokens, (long long)p.B, checksum);
  return 0;
}

int main() {
  const std::vector<int32_t> t13 = {1, 4, 16, 36, 64, 144, 256, 400, 576, 1024, 1600, 2304, 4096};
  const std::vector<int32_t> t6 = {1, 4, 9, 16, 25, 36};
  const std::vector<int32_t> t2 = {3, 5};
  int bad = 0;
  for (int variant = 0; variant < 4; ++variant) {
    bad |= run_case(32, 16, t13, 3, variant, 10);
    bad |= run_case(40, 32, t13, 3, variant, 20);
    bad |= run_case(3, 5, t6, 2, variant, 2);
    bad |= run_case(1, 1, t6, 0, variant, 3);
    bad |= run_case(2, 2, t2, 0, variant, 1);
    bad |= run_case(4, 4, t6, 4, variant, 50);  // budget below the sinks -> EBUDGET path
  }
  if (bad) std::printf("FAILED code %d\n", bad);
  return bad;
}

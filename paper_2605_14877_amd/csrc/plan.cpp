// Host planner: head ranking (Eq. 3-4), budget rule (Eq. 5), removal-order
// optimisation (Alg. 1 with the cache accounting of Alg. 2 / App. A), and the
// static memory layout the kernels run on.  Pure integer work apart from the
// fp64 sums that rank the heads.  No HIP calls in this file.
#include "plan.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <deque>
#include <numeric>

namespace heatkv {

static thread_local std::string g_last_error;

void set_error(const std::string& msg) { g_last_error = msg; }
int fail(int code, const std::string& msg) {
  g_last_error = msg;
  return code;
}
const char* last_error_cstr() { return g_last_error.c_str(); }

int check_shape(const heatkv_shape* s) {
  if (!s) return fail(HEATKV_EINVAL, "shape is null");
  if (!s->t) return fail(HEATKV_EINVAL, "shape.t is null");
  if (s->L < 1 || s->H < 1 || s->batch < 1) return fail(HEATKV_EINVAL, "L, H, batch must be >= 1");
  if (s->K < 1 || s->K > HEATKV_MAX_SCALES) return fail(HEATKV_EINVAL, "K out of range");
  if (s->dtype != HEATKV_F32 && s->dtype != HEATKV_BF16) return fail(HEATKV_EINVAL, "unknown dtype");
  if (s->d != 64 && s->d != 128) return fail(HEATKV_EINVAL, "head dimension must be 64 or 128");
  int64_t total = 0;
  for (int k = 0; k < s->K; ++k) {
    if (s->t[k] < 1) return fail(HEATKV_EINVAL, "t[k] must be >= 1");
    total += s->t[k];
  }
  if (total * s->H > (int64_t(1) << 30)) return fail(HEATKV_EINVAL, "sequence too long");
  return HEATKV_OK;
}

int init_shape(heatkv_plan* p, const heatkv_shape* s) {
  int rc = check_shape(s);
  if (rc) return rc;
  p->L = s->L;
  p->H = s->H;
  p->d = s->d;
  p->K = s->K;
  p->batch = s->batch;
  p->dtype = s->dtype;
  p->T = s->L * s->H;
  p->t.assign(s->t, s->t + s->K);
  p->c.resize(s->K);
  int32_t acc = 0;
  for (int k = 0; k < s->K; ++k) {
    acc += p->t[k];
    p->c[k] = acc;
  }
  return HEATKV_OK;
}

namespace {

// Stable ascending order of the heads by an fp64 score; ties keep the flat head id order.
std::vector<int32_t> rank_heads(const std::vector<double>& score) {
  std::vector<int32_t> order(score.size());
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return score[a] < score[b]; });
  return order;
}

// Head scores that the orders are built from: score[i][head] for source scale i in [s, K-1), the
// un-normalised sums of Eq. 4 (scale-dependent) or Eq. 3 (binary: the same sum for every i); fp64, tau ascending.
void head_scores(int K, int T, int s, bool binary, const float* beta, std::vector<std::vector<double>>& score) {
  auto b = [&](int head, int k1, int k2) { return double(beta[(size_t(head) * K + k1) * K + k2]); };
  score.assign(K, {});
  if (binary) {
    std::vector<double> sc(T, 0.0);
    for (int head = 0; head < T; ++head)
      for (int tau = s; tau < K - 1; ++tau) sc[head] += b(head, K - 1, tau);
    for (int i = s; i < K - 1; ++i) score[i] = sc;
  } else {
    for (int i = s; i < K - 1; ++i) {
      score[i].assign(T, 0.0);
      for (int head = 0; head < T; ++head)
        for (int tau = i + 1; tau < K; ++tau) score[i][head] += b(head, tau, i);
    }
  }
}

struct Candidate {
  int32_t layer, scale, rank, head;
  int64_t weight;  // tokens its early removal takes out of a not-yet-run layer
};

}  // namespace

int build_sets(heatkv_plan* p, const float* beta) {
  const int K = p->K, L = p->L, H = p->H, T = p->T, s = p->sinks;
  const bool binary = (p->variant & 1) != 0, naive = (p->variant & 2) != 0;
  const int64_t cs = s > 0 ? p->c[s - 1] : 0;
  const int64_t B = p->B;

  // Eq. 5 in integers.
  p->N.assign(K > 1 ? K - 1 : 0, 0);
  for (int k = s; k < K - 1; ++k) {
    const int64_t num = int64_t(T) * p->c[k] - B, den = p->c[k] - cs;
    int64_t n = num <= 0 ? 0 : (num + den - 1) / den;
    if (n > T) return fail(HEATKV_EBUDGET, "budget is smaller than the sink scales of all heads");
    p->N[k] = int32_t(n);
  }
  if (B < int64_t(T) * cs) return fail(HEATKV_EBUDGET, "budget is smaller than the sink scales of all heads");

  // Orders.  beta[l][h][k1][k2]; sums in fp64, tau ascending.
  std::vector<std::vector<double>> score;
  head_scores(K, T, s, binary, beta, score);
  p->orders.assign(K, {});
  for (int i = s; i < K - 1; ++i) {
    if (binary && i > s) p->orders[i] = p->orders[s];
    else p->orders[i] = rank_heads(score[i]);
  }

  const size_t KT = size_t(K) * T;
  p->G.assign(size_t(K) * KT, 0);
  p->E.assign(size_t(K) * KT, 0);
  p->A.assign(size_t(K) * KT, 0);
  auto at = [&](std::vector<uint8_t>& S, int k, int i, int head) -> uint8_t& { return S[size_t(k) * KT + size_t(i) * T + head]; };

  std::vector<int64_t> done(L), todo(L);
  for (int k = 0; k < K - 1; ++k) {
    // G_k: prefix of length N_k of every order O_i, i <= k (binary: of the one order, all scales).
    std::vector<Candidate> cand;
    if (k >= s && p->N[k] > 0) {
      if (binary) {
        for (int r = 0; r < p->N[k]; ++r) {
          const int head = p->orders[s][r];
          const bool fresh = !(k > 0 && at(p->G, k - 1, s, head));
          for (int i = s; i < K - 1; ++i) at(p->G, k, i, head) = 1;
          if (fresh) cand.push_back({head / H, 0, r, head, int64_t(p->c[k]) - cs});
        }
      } else {
        for (int i = s; i <= k; ++i)
          for (int r = 0; r < p->N[k]; ++r) {
            const int head = p->orders[i][r];
            at(p->G, k, i, head) = 1;
            if (!(k > 0 && at(p->G, k - 1, i, head))) cand.push_back({head / H, i, r, head, int64_t(p->t[i])});
          }
      }
    }
    std::sort(cand.begin(), cand.end(), [](const Candidate& a, const Candidate& c2) {
      if (a.layer != c2.layer) return a.layer > c2.layer;
      if (a.scale != c2.scale) return a.scale > c2.scale;
      return a.rank < c2.rank;
    });

    // Cache size per layer with G_k applied (layers that have run) and with only
    // G_{k-1} applied (layers still to run); early removals lower the latter.
    std::fill(done.begin(), done.end(), 0);
    std::fill(todo.begin(), todo.end(), 0);
    for (int head = 0; head < T; ++head) {
      int64_t dn = cs, td = cs;
      for (int i = s; i <= k; ++i) {
        if (!at(p->G, k, i, head)) dn += p->t[i];
        if (!(k > 0 && at(p->G, k - 1, i, head))) td += p->t[i];
      }
      done[head / H] += dn;
      todo[head / H] += td;
    }
    size_t next = 0;
    auto pop = [&]() {
      const Candidate& cd = cand[next++];
      if (binary) {
        for (int i = s; i < K - 1; ++i) at(p->E, k, i, cd.head) = 1;
      } else {
        at(p->E, k, cd.scale, cd.head) = 1;
      }
      todo[cd.layer] -= cd.weight;
      return cd.layer;
    };
    if (naive) {
      while (next < cand.size()) pop();
    }
    for (int l = 0; l < L; ++l) {
      int64_t M = 0;
      for (int lp = 0; lp < L; ++lp) M += lp <= l ? done[lp] : todo[lp];
      while (M > B) {
        if (next >= cand.size()) return fail(HEATKV_EBUDGET, "early pruning cannot reach the budget");
        const int64_t w = cand[next].weight;
        if (pop() > l) M -= w;
      }
    }
    // A_k = G_{k-1} u E_k
    for (int i = 0; i < K; ++i)
      for (int head = 0; head < T; ++head)
        at(p->A, k, i, head) = uint8_t((k > 0 && at(p->G, k - 1, i, head)) || at(p->E, k, i, head));
  }
  // Last scale: nothing is appended any more, so only the removals already decided apply.
  if (K >= 2) std::memcpy(&p->A[size_t(K - 1) * KT], &p->G[size_t(K - 2) * KT], KT);

  p->retained.assign(size_t(K) * T, 0);
  for (int k = 0; k < K; ++k)
    for (int head = 0; head < T; ++head) {
      uint32_t m = 0;
      for (int i = 0; i < k; ++i)
        if (i < s || !at(p->A, k, i, head)) m |= 1u << i;
      p->retained[size_t(k) * T + head] = m;
    }
  return HEATKV_OK;
}

int rank_scores(const heatkv_shape* shape, const float* beta, int sinks, int variant, double* scores) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!beta || !scores) return fail(HEATKV_EINVAL, "null pointer");
  const int K = shape->K, T = shape->L * shape->H;
  if (sinks < 0 || sinks > K - 2) return fail(HEATKV_EINVAL, "sinks out of range");
  if (variant < 0 || variant > 3) return fail(HEATKV_EINVAL, "unknown variant");
  std::vector<std::vector<double>> score;
  head_scores(K, T, sinks, (variant & 1) != 0, beta, score);
  for (int i = 0; i < K; ++i)
    for (int head = 0; head < T; ++head) scores[size_t(i) * T + head] = score[i].empty() ? 0.0 : score[i][head];
  return HEATKV_OK;
}

int rank_dispersion(const heatkv_shape* shape, const float* betas, int runs, int sinks, int variant,
                    double* dispersion) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!betas || !dispersion) return fail(HEATKV_EINVAL, "null pointer");
  if (runs < 1) return fail(HEATKV_EINVAL, "runs must be >= 1");
  const int K = shape->K, T = shape->L * shape->H;
  if (sinks < 0 || sinks > K - 2) return fail(HEATKV_EINVAL, "sinks out of range");
  if (variant < 0 || variant > 3) return fail(HEATKV_EINVAL, "unknown variant");
  const bool binary = (variant & 1) != 0;
  const size_t table = size_t(T) * K * K;
  // pos[i][run][head] = rank position of the head in that run's order O_i
  std::vector<std::vector<int32_t>> pos(K);
  for (int r = 0; r < runs; ++r) {
    std::vector<std::vector<double>> score;
    head_scores(K, T, sinks, binary, betas + size_t(r) * table, score);
    std::vector<int32_t> first;
    for (int i = sinks; i < K - 1; ++i) {
      if (pos[i].empty()) pos[i].assign(size_t(runs) * T, 0);
      std::vector<int32_t> order = (binary && i > sinks) ? first : rank_heads(score[i]);
      if (i == sinks) first = order;
      for (int rank = 0; rank < T; ++rank) pos[i][size_t(r) * T + order[rank]] = rank;
    }
  }
  for (int i = 0; i < K; ++i) dispersion[i] = 0.0;
  for (int i = sinks; i < K - 1; ++i) {
    double total = 0.0;
    for (int head = 0; head < T; ++head) {
      int64_t sum = 0;
      for (int r = 0; r < runs; ++r) sum += pos[i][size_t(r) * T + head];
      const double mean = double(sum) / runs;
      double var = 0.0;
      for (int r = 0; r < runs; ++r) {
        const double dlt = pos[i][size_t(r) * T + head] - mean;
        var += dlt * dlt;
      }
      total += std::sqrt(var / runs);
    }
    dispersion[i] = total / T;
  }
  return HEATKV_OK;
}

int load_pattern(heatkv_plan* p, const uint8_t* present) {
  const int K = p->K, T = p->T;
  p->retained.assign(size_t(K) * T, 0);
  for (int k = 0; k < K; ++k)
    for (int head = 0; head < T; ++head) {
      uint32_t m = 0;
      for (int i = 0; i < K; ++i) {
        const bool on = present[(size_t(k) * T + head) * K + i] != 0;
        if (on && i >= k) return fail(HEATKV_EINVAL, "present[k][..][i] set for i >= k");
        if (on) m |= 1u << i;
      }
      if (k > 0) {
        const uint32_t prev = p->retained[size_t(k - 1) * T + head];
        const uint32_t older = m & ((1u << (k - 1)) - 1u);
        if (older & ~prev) return fail(HEATKV_EINVAL, "a scale absent at scale k-1 is present at scale k");
      }
      p->retained[size_t(k) * T + head] = m;
    }
  return HEATKV_OK;
}

namespace {

constexpr int32_t kCopyChunkRows = 128;

// Places the layer regions of successive scales in one arena of `cap` rows as a
// FIFO: region (k+1,l) is allocated, then region (k,l) is released, in
// generation order.  A region never straddles the end of the arena.
bool place_regions(heatkv_plan* p, int64_t cap) {
  const int K = p->K, L = p->L;
  struct Live {
    int64_t base, size;
  };
  std::deque<Live> live;
  int64_t tail = 0;
  std::fill(p->region_base.begin(), p->region_base.end(), 0);
  for (int k = 0; k + 1 < K; ++k)
    for (int l = 0; l < L; ++l) {
      const int64_t S = p->region_size[p->idx(k + 1, l)];
      if (S > 0) {
        int64_t base;
        if (live.empty()) {
          base = 0;
          if (S > cap) return false;
        } else {
          const bool wrapped = live.front().base > live.back().base;
          if (!wrapped) {
            if (tail + S <= cap) base = tail;
            else if (S <= live.front().base) base = 0;
            else return false;
          } else {
            if (tail + S <= live.front().base) base = tail;
            else return false;
          }
        }
        p->region_base[p->idx(k + 1, l)] = base;
        live.push_back({base, S});
        tail = base + S;
      }
      if (p->region_size[p->idx(k, l)] > 0) live.pop_front();
    }
  return true;
}

}  // namespace

int derive_layout(heatkv_plan* p) {
  const int K = p->K, L = p->L, H = p->H, T = p->T;
  const size_t n3 = size_t(K) * L * H, n2 = size_t(K) * L;
  p->run_len.assign(n3, 0);
  p->run_row.assign(n3, 0);
  p->head_order.assign(n3, 0);
  p->region_size.assign(n2, 0);
  p->region_base.assign(n2, 0);
  p->max_len.assign(n2, 0);

  for (int k = 0; k < K; ++k)
    for (int l = 0; l < L; ++l) {
      int64_t sum = 0;
      int32_t mx = 0;
      for (int h = 0; h < H; ++h) {
        const uint32_t m = p->retained[size_t(k) * T + l * H + h];
        int32_t len = 0;
        for (int i = 0; i < k; ++i)
          if (m >> i & 1u) len += p->t[i];
        p->run_len[p->idx(k, l, h)] = len;
        sum += len;
        mx = std::max(mx, len);
      }
      p->region_size[p->idx(k, l)] = sum;
      p->max_len[p->idx(k, l)] = mx;
      int32_t* ord = &p->head_order[p->idx(k, l, 0)];
      std::iota(ord, ord + H, 0);
      const int32_t* len = &p->run_len[p->idx(k, l, 0)];
      std::stable_sort(ord, ord + H, [&](int32_t a, int32_t b) { return len[a] > len[b]; });
    }

  // Smallest arena (searched upward from the peak of live + incoming rows) in which the FIFO fits.
  int64_t lower = 0, max_region = 0, live = 0;
  for (int k = 0; k + 1 < K; ++k)
    for (int l = 0; l < L; ++l) {
      const int64_t S = p->region_size[p->idx(k + 1, l)];
      max_region = std::max(max_region, S);
      lower = std::max(lower, live + S);
      live += S - p->region_size[p->idx(k, l)];
    }
  lower = std::max<int64_t>(lower, 1);
  const int64_t step = std::max<int64_t>(1, (max_region + 31) / 32);
  int64_t cap = lower;
  bool ok = false;
  for (int tries = 0; tries < 4096; ++tries, cap += step)
    if ((ok = place_regions(p, cap))) break;
  if (!ok) return fail(HEATKV_ENOMEM, "no arena placement found");
  if (cap * p->batch > (int64_t(1) << 31) - 1) return fail(HEATKV_EINVAL, "arena rows exceed 2^31");
  p->arena_tokens = cap;

  for (int k = 0; k < K; ++k)
    for (int l = 0; l < L; ++l) {
      int64_t row = p->region_base[p->idx(k, l)];
      for (int h = 0; h < H; ++h) {
        p->run_row[p->idx(k, l, h)] = int32_t(row);
        row += p->run_len[p->idx(k, l, h)];
      }
    }

  // Append descriptors: the move from the scale-k runs (plus the new scale) to the scale-(k+1) runs.
  p->descs.clear();
  p->desc_begin.assign(n2, 0);
  p->desc_count.assign(n2, 0);
  for (int k = 0; k + 1 < K; ++k)
    for (int l = 0; l < L; ++l) {
      const size_t begin = p->descs.size();
      for (int h = 0; h < H; ++h) {
        const uint32_t now = p->retained[size_t(k) * T + l * H + h];
        const uint32_t nxt = p->retained[size_t(k + 1) * T + l * H + h];
        int32_t dst = p->run_row[p->idx(k + 1, l, h)];
        int32_t src = p->run_row[p->idx(k, l, h)];
        std::vector<heatkv::CopyDesc> segs;
        for (int i = 0; i <= k; ++i) {
          const bool keep = (nxt >> i & 1u) != 0;
          if (i < k) {
            const bool have = (now >> i & 1u) != 0;
            if (keep) {
              if (!segs.empty() && segs.back().src_kind == 0 && segs.back().src_row + segs.back().nrows == src)
                segs.back().nrows += p->t[i];
              else
                segs.push_back({dst, src, p->t[i], 0});
              dst += p->t[i];
            }
            if (have) src += p->t[i];
          } else if (keep) {
            segs.push_back({dst, h * p->t[k], p->t[k], 1});
            dst += p->t[k];
          }
        }
        for (const auto& sg : segs)
          for (int32_t o = 0; o < sg.nrows; o += kCopyChunkRows)
            p->descs.push_back({sg.dst_row + o, sg.src_row + o, std::min(kCopyChunkRows, sg.nrows - o), sg.src_kind});
      }
      p->desc_begin[p->idx(k, l)] = int64_t(begin);
      p->desc_count[p->idx(k, l)] = int32_t(p->descs.size() - begin);
    }
  return HEATKV_OK;
}

}  // namespace heatkv

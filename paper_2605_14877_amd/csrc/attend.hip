// Next-scale attention over the ragged per-head KV cache (Sec. 3.1 attention rows,
// Sec. 3.3 for which prior scales a head still holds).
//
// For head (b,h) the keys are the head's run of retained rows in the arena
// followed by the t_k rows of the current scale; queries are the t_k rows of
// the current scale.  Both kernels walk this virtual key sequence in tiles,
// keep running row maxima and row sums in fp32 (online softmax) and normalise
// once at the end.
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "copy_rows.h"
#include "device_util.h"
#include "kernels.h"
#include "tile_lds.h"

namespace heatkv {

namespace {

struct AttendParams {
  int H, batch, t_k;
  long long arena_tokens;
  const HeadWork* work;
  // uniform_len >= 0: every head of the layer holds a run of that many rows, head h's run starts at row
  // uniform_row0 + h * uniform_len, and (batch row, head) pairs are taken in index order: a workgroup then knows
  // all its addresses from its id and the kernel arguments, and its first fetches do not wait for a table read.
  int uniform_len, uniform_row0;
  const void *q, *k_cur, *v_cur, *k_arena, *v_arena;
  void* out;
  float sm_scale;
  int n_qtiles;
  // Workgroups with blockIdx.x >= attend_blocks run the fused cache update (copy descriptor, batch entry).
  // They sit at the end of the grid on purpose: there they fill the slots that the last attention workgroups
  // leave one by one.  Spread through the grid instead, their memory traffic lengthened the latency of the
  // attention workgroups' tile fetches and the launch became up to 1.4x slower.
  int attend_blocks;
  int ndesc;
  CopyParams copy;
};

// ---------------------------------------------------------------------------
// bf16, d = 128 or 64: matrix-core kernel (the description takes d = 128: rows of 256 bytes).
//
// Workgroup = 4 wavefronts x 32 queries, two workgroups per compute unit.  The
// keys of a head are walked in 64-row tiles, first the current scale (dense
// tensor), then the head's retained run in the arena (attention does not depend
// on key order, and each segment is then one contiguous range, so a tile's
// addresses are a wavefront-uniform base plus a fixed per-lane offset).
//
// Tiles go from HBM straight into LDS (global_load_lds, no registers, no LDS
// store instructions), double-buffered with one barrier per tile.  A tile is
// stored row-major, 256 bytes per row, unpadded; the 16-byte chunks of a row are
// XOR-swizzled with the row number (the lane that fills an LDS slot simply
// fetches the matching global chunk), K tiles and V tiles each with the pattern
// that keeps their read instruction free of bank conflicts (tile_lds.h holds the
// format; the calibration kernel and the measurement probes share it).
//
// Scores are produced transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: K
// rows are the A operand straight from LDS, Q stays in registers as the B operand.
// One lane then owns one query column: row maxima and sums are in-register
// reductions plus one exchange between the wavefront halves, and the bf16
// probabilities already sit in the B-operand layout of O^T += V^T P^T.  V^T comes
// out of the row-major V tile with the transposing LDS read; the order of keys
// inside a 16-key MFMA step is permuted identically on both operands.
// ---------------------------------------------------------------------------
constexpr int BM = 128;              // queries per workgroup
constexpr int BN = tile::ROWS;       // keys per tile
constexpr int TILE_BYTES_D128 = tile::BYTES;  // 64 rows x 256 bytes

extern __shared__ __attribute__((aligned(1024))) char attend_dynamic_lds[];

// KS = number of key streams.  KS = 1: the workgroup described above.  KS = 2, for launches that give every
// compute unit at most one workgroup (few heads, small batch): 8 wavefronts, one workgroup per unit; wavefronts
// 4-7 take the same 128 queries as 0-3 but every other key tile (stream g walks tiles g, g + 2, ...), each
// stream with its own pair of tile stages (128 KB of dynamic LDS), and at the end stream 1 hands its partial
// output, row sums and references to stream 0 through LDS.  The unit then runs two wavefronts per SIMD, as it
// does when two workgroups share it, without a second pass over HBM.
//
// FP8: the arenas hold FP8 E4M3 codes, 128 bytes per row (single-stream instances only).  A tile of the retained run
// lands as it is (8 KB) in a landing buffer behind the tile stages, one for K and one for V, and at the top of the
// step that first needs it the whole workgroup rewrites it as a bf16 tile in its stage (exact: every E4M3 value is
// a bf16 value), with one more barrier; from there on the step is the same.  Current-scale tiles are bf16 and go
// straight to their stage.  80 KB of LDS per workgroup: two workgroups still share a compute unit.
//
// D: head dimension, 128 or 64 (rows of 256 or 128 bytes, tiles of 16 or 8 KB, 8 or 4 MFMA steps per score block and
// 4 or 2 accumulator blocks; the single-stream, bf16-cache instance only).
//
// QS = 2, for launches that keep every compute unit busy for rounds of long walks: 8 wavefronts, one workgroup
// per unit, 256 queries per workgroup; wavefronts 4-7 take the next 128 queries against the SAME key tiles, which
// all eight wavefronts copy together (two instead of four copies per wavefront and tile).  A K/V tile then enters
// the LDS once per 256 queries instead of once per 128: the copies, which cost the single-set instance 14-18 % of
// its time at these scales whether they come from HBM or from L2, are halved per FLOP.  The two wavefronts of a SIMD
// now pass the same barriers and so run the same part of the step at the same time; that costs nothing because
// every slot of the hand-ordered step below mixes matrix and vector work (with the compiler's own order, score
// MFMAs clustered apart from the exponentials, the same instance gained 1 % instead of 4-6 %).
template <int KS, bool FP8, int D, int QS = 1>
__global__ __launch_bounds__(256 * KS * QS, (KS == 1 && QS == 1) ? 2 : 1) void attend_bf16_kernel(AttendParams p) {
  static_assert(KS == 1 || KS == 2, "one or two key streams");
  static_assert(QS == 1 || QS == 2, "one or two query sets");
  static_assert(!(FP8 && KS == 2), "the 8-bit cache path has one key stream");
  static_assert(D == 128 || (D == 64 && KS == 1 && !FP8), "d = 64: single stream, bf16 cache rows");
  static_assert(QS == 1 || (KS == 1 && D == 128), "two query sets: single stream, d = 128");
  constexpr int NW = 4 * QS;  // wavefronts that share the copying of a tile
  constexpr int ROW_BYTES = 2 * D;            // one bf16 row
  constexpr int TILE_BYTES = BN * ROW_BYTES;  // 16 KB (d = 128) or 8 KB (d = 64)
  constexpr int CPR = ROW_BYTES / 16;         // 16-byte chunks per row
  constexpr int NK = D / 16, NV = D / 32;     // MFMA steps of a score block, accumulator blocks of 32 columns
  constexpr bool kStaticLds = KS == 1 && !FP8;
  __shared__ __attribute__((aligned(1024))) char lds_static[kStaticLds ? 2 : 1][2][kStaticLds ? TILE_BYTES : 16];
  // [stream * 2 + stage][K,V]; 64 KB are static, anything more exceeds the static limit and comes as dynamic LDS
  char(*lds)[2][TILE_BYTES] = kStaticLds ? reinterpret_cast<char(*)[2][TILE_BYTES]>(&lds_static[0][0][0])
                                         : reinterpret_cast<char(*)[2][TILE_BYTES]>(attend_dynamic_lds);
  char* const raw_k = reinterpret_cast<char*>(lds) + 4 * TILE_BYTES;  // FP8 only: landing buffers, 8 KB each
  char* const raw_v = raw_k + tile::RAW8_BYTES;

  if (static_cast<int>(blockIdx.x) >= p.attend_blocks) {  // fused append: a plain row copy by 256 lanes
    const int j = blockIdx.x - p.attend_blocks;
    if ((KS == 1 && QS == 1) || threadIdx.x < 256) copy_rows_block(p.copy, j % p.ndesc, j / p.ndesc);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform, kept in a scalar register
  const int g = KS == 1 ? 0 : wave_all >> 2;                      // key stream of this wavefront
  const int qs = QS == 1 ? 0 : wave_all >> 2;                     // query set of this wavefront
  const int wave = wave_all & 3;                                  // its place among the four of the stream / set
  const int lw = QS == 1 ? wave : wave_all;                       // its place among the NW that copy a tile
  const int n = lane & 31, hl = lane >> 5;

  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  All query tiles of one
  // (batch row, head) pair read the same K/V, so they are given ids that land on one XCD; pairs are dealt
  // to XCDs in order of decreasing run length, alternating direction, which balances the work between XCDs.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int turn = slot / p.n_qtiles;  // pairs are dealt to the XCDs back and forth (0..7, 7..0, 0..7, ...)
  const int pair = turn * 8 + ((turn & 1) ? 7 - xcd : xcd);
  if (pair >= p.H * p.batch) return;
  const int qt = slot % p.n_qtiles;
  const int b = pair % p.batch;
  int h, n_prior, run_row;
  if (p.uniform_len >= 0) {
    h = pair / p.batch;
    n_prior = p.uniform_len;
    run_row = p.uniform_row0 + h * p.uniform_len;
  } else {
    const HeadWork hw = p.work[pair / p.batch];  // one 16-byte record: head, first row and length of its run
    h = hw.head;
    n_prior = hw.run_len;
    run_row = hw.run_row;
  }

  const int t_k = p.t_k;
  const long long cur_off = (static_cast<long long>(b) * p.H + h) * t_k * D;
  constexpr int PRIOR_ROW_BYTES = FP8 ? tile::RAW8_ROW_BYTES : ROW_BYTES;
  constexpr int PRIOR_TILE_BYTES = BN * PRIOR_ROW_BYTES;
  const long long run_off = (static_cast<long long>(b) * p.arena_tokens + run_row) * PRIOR_ROW_BYTES;
  const char* k_prior = static_cast<const char*>(p.k_arena) + run_off;
  const char* v_prior = static_cast<const char*>(p.v_arena) + run_off;
  const char* k_cur = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.k_cur) + cur_off);
  const char* v_cur = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.v_cur) + cur_off);

  // Q as B operand: lane (n, hl) holds Q[row][16*ks + 8*hl .. +7] for ks = 0..7.
  const int q_row0 = qt * (BM * QS) + qs * BM + wave * 32;  // first query row of this wavefront
  const int q_row = q_row0 + n;
  bf16x8 qreg[NK];
  {
    const int ld = q_row < t_k ? q_row : t_k - 1;
    const bf16_t* qp = static_cast<const bf16_t*>(p.q) + cur_off + static_cast<long long>(ld) * D + 8 * hl;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  // Tile schedule: tiles [0, tiles_cur) cover the current scale, the rest the retained run.
  const int tiles_cur = (t_k + BN - 1) / BN;
  const int tiles_all = tiles_cur + (n_prior + BN - 1) / BN;
  // Step j of stream g works on tile KS j + g; all streams make steps_all steps (the barriers are shared), a
  // stream whose last step has no tile sits it out.
  const int steps_all = (tiles_all + KS - 1) / KS;
  auto has_tile = [&](int j) { return KS == 1 || KS * j + g < tiles_all; };

  // Loader and reader offsets of the shared tile format.  The copy HBM -> LDS is issued as raw global_load_lds
  // instructions (tile::issue_full / issue_ragged): the compiler then does not see an LDS store it would have to
  // order against the tile reads of the other buffer (it would wait for the whole prefetch in the middle of the
  // math).  Ordering is explicit instead: s_waitcnt vmcnt(0) and the workgroup barrier at the top of every step.
  const int ld_off_k = tile::loader_off_k<ROW_BYTES>(lw, lane);
  const int ld_off_v = tile::loader_off_v<ROW_BYTES>(lw, lane);
  const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<unsigned long long>(
      (__attribute__((address_space(3))) char*)(&lds[0][0][0]))) + g * (4 * TILE_BYTES);
  int k_off[NK], v_off[NV];
  tile::reader_off_k<ROW_BYTES>(lane, k_off);
  tile::reader_off_v<ROW_BYTES>(lane, v_off);

  f32x16 o[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = p.sm_scale * kLog2e;
  // The running reference m_run of a row is only raised when the tile maximum exceeds it by more than
  // kSlack in the exponent (base 2): probabilities are then at most 2^kSlack, far inside fp32/bf16 range,
  // the final division by the row sum makes the result independent of the reference, and the expensive
  // rescaling of the accumulators happens a handful of times per row instead of every few tiles.
  constexpr float kSlack = 8.f;
  const float slack_raw = kSlack / c;
  const bf16x2 ones = {static_cast<bf16_t>(1.f), static_cast<bf16_t>(1.f)};

  // ---- software-pipelined tile loop --------------------------------------------------------------
  // Step `it` computes the scores of tile it+1 (matrix cores) while it turns the scores of tile `it` into
  // probabilities (vector ALU) and accumulates P V for tile `it`.  K tiles are therefore fetched one tile
  // further ahead than V tiles: at the top of step `it` the copies K(it+1) and V(it) must have landed.
  auto issue_k = [&](int j, int buf) {
    const int it = KS * j + g;
    const bool prior = it >= tiles_cur;
    const int local = prior ? it - tiles_cur : it;
    const int left = (prior ? n_prior : t_k) - local * BN;
    if (FP8 && prior) {  // codes land in the K landing buffer; the step that needs the tile converts it
      tile::issue_raw8<NW>(lds_base + 4 * TILE_BYTES, lw, lane, left, k_prior + static_cast<long long>(local) * PRIOR_TILE_BYTES);
      return;
    }
    const char* kb = (prior ? k_prior : k_cur) + static_cast<long long>(local) * TILE_BYTES;
    const unsigned kd = lds_base + buf * (2 * TILE_BYTES);
    // Two separate statements under a workgroup-uniform branch: the full-tile path has no per-lane arithmetic.
    if (left >= BN)
      tile::issue_full<ROW_BYTES, NW>(kd, lw, ld_off_k, kb);
    else
      tile::issue_ragged<false, ROW_BYTES, NW>(kd, lw, lane, left, kb);
  };
  auto issue_v = [&](int j, int buf) {
    const int it = KS * j + g;
    const bool prior = it >= tiles_cur;
    const int local = prior ? it - tiles_cur : it;
    const int left = (prior ? n_prior : t_k) - local * BN;
    if (FP8 && prior) {
      tile::issue_raw8<NW>(lds_base + 4 * TILE_BYTES + tile::RAW8_BYTES, lw, lane, left,
                           v_prior + static_cast<long long>(local) * PRIOR_TILE_BYTES);
      return;
    }
    const char* vb = (prior ? v_prior : v_cur) + static_cast<long long>(local) * TILE_BYTES;
    const unsigned vd = lds_base + buf * (2 * TILE_BYTES) + TILE_BYTES;
    if (left >= BN)
      tile::issue_full<ROW_BYTES, NW>(vd, lw, ld_off_v, vb);
    else
      tile::issue_ragged<true, ROW_BYTES, NW>(vd, lw, lane, left, vb);
  };

  // S^T = K Q^T for the 64 keys of the K tile in buffer `buf` x this wavefront's 32 queries.
  // s[cb][r] is key 32*cb + 8*(r/4) + 4*hl + r%4 of the tile, query column n.
  auto scores = [&](f32x16 (&s)[2], auto buf_tag) {
    constexpr int buf = decltype(buf_tag)::value;
    const char* kt = lds[2 * g + buf][0];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kt + cb * 32 * ROW_BYTES + k_off[ks]);
        s[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s[cb], 0, 0, 0);
      }
  };
  // Folds the maximum of a tile's scores (this lane's 32 of them) into the running reference and, rarely,
  // rescales what has been accumulated so far.
  auto raise = [&](float mx) {
    mx = max_halves(mx);
    if (__any(mx > m_run + slack_raw)) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2((m_run - m_new) * c);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
    }
  };
  auto lane_max = [&](const f32x16 (&s)[2]) {
    float mx = s[0][0];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[cb][r]);
    return mx;
  };
  // Masks the ragged tail of the stream's tile j (keys past the end of the scale or of the run get -inf);
  // returns whether there was one.
  auto mask_tail = [&](int j, f32x16 (&s)[2]) {
    const int it = KS * j + g;
    const bool prior = it >= tiles_cur;
    const int left = (prior ? n_prior : t_k) - (prior ? it - tiles_cur : it) * BN;
    if (left >= BN) return false;  // workgroup-uniform and rare: kept a branch
    // Register r of block cb holds key 32 cb + 8 (r / 4) + r % 4 + 4 hl: compared as a compile-time constant
    // against one per-lane limit, formed here and hidden from the optimiser so that it is not turned back into
    // 32 per-lane key numbers that would live in registers across the whole tile loop (nor into 32 selects).
    int lim = left - 4 * hl;
    asm volatile("; ragged tile mask" : "+v"(lim)::"memory");
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * cb + 8 * (r >> 2) + (r & 3) >= lim) s[cb][r] = -INFINITY;
    return true;
  };
  // Masks the tail of tile j and folds its row maxima into the running reference.
  auto settle = [&](int j, f32x16 (&s)[2]) {
    mask_tail(j, s);
    raise(lane_max(s));
  };
  // P^T = 2^(S^T c - m c) in bf16, 16 keys at a time, each chunk feeding O^T += V^T P^T at once.  The row
  // sum is taken over the rounded probabilities, pairwise, with the bf16 dot-product instruction.
  union VOperand {
    struct {
      s16x4 lo, hi;
    } s;
    bf16x8 v;
  };
  auto accumulate = [&](const f32x16 (&s)[2], auto buf_tag) {
    constexpr int buf = decltype(buf_tag)::value;
    const char* vt = lds[2 * g + buf][1];
    const float mc = m_run * c;
#pragma unroll
    for (int chunk = 0; chunk < 4; ++chunk) {
      const int cb = chunk >> 1, ks = chunk & 1;
      VOperand va[NV];
#pragma unroll
      for (int dblk = 0; dblk < NV; ++dblk) {
        const char* base = vt + 16 * chunk * ROW_BYTES + v_off[dblk];
        va[dblk].s.lo = lds_read_tr16(reinterpret_cast<const bf16_t*>(base));
        va[dblk].s.hi = lds_read_tr16(reinterpret_cast<const bf16_t*>(base + 8 * ROW_BYTES));
      }
      union {
        bf16x8 v;
        bf16x2 h[4];
      } pb;
#pragma unroll
      for (int j = 0; j < 8; ++j) pb.v[j] = static_cast<bf16_t>(fast_exp2(fmaf(s[cb][8 * ks + j], c, -mc)));
#pragma unroll
      for (int j = 0; j < 4; ++j) l_run = __builtin_amdgcn_fdot2_f32_bf16(pb.h[j], ones, l_run, false);
#pragma unroll
      for (int dblk = 0; dblk < NV; ++dblk)
        o[dblk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dblk].v, pb.v, o[dblk], 0, 0, 0);
    }
  };

  // The steady-state step in one piece: scores of the next tile into s_out, P V of this tile from s_in, with the
  // order of issue fixed by hand.  Left to itself the compiler clusters the score MFMAs at the K reads that feed
  // them, back to back, and the exponentials elsewhere; a wavefront issues in order, so an MFMA waiting for the
  // matrix pipe holds back the vector work that could run in the shadow of the one before.  Here the step is a
  // sequence of 32 slots, one MFMA each followed by its share of vector and LDS work; scheduling fences keep the
  // slots apart and the MFMA at the head of its slot:
  //   S(g), g = 0..3: the NK/4 K-steps of the score product that go with chunk g (both 32-key blocks)
  //   A(g): P V for the 16 keys of chunk g (NV MFMAs)
  //   order S(0) A(0) S(1) A(1) S(2) A(2) S(3) A(3).  P(0) is computed in the slots of S(0), P(g+1) in those of
  //   A(g) and S(g+1), the row maxima of the new scores in those of A(3); the K operands of S(g+1) are read in the
  //   slots of S(g), the V operands of A(g+1) in those of A(g): every operand a whole phase before its MFMA (those
  //   of S(0) and A(0), which only exist after the barrier, in preload() and in the slots of S(0)).
  // Returns this lane's maximum over the new scores (before any tail mask).
  auto step_math = [&](const f32x16 (&s_in)[2], f32x16 (&s_out)[2], const bf16x8 (&k0)[2], auto kb1, auto vb0) {
    constexpr int KPC = NK / 4;          // K-steps per phase S
    constexpr int NS = 2 * KPC;          // slots of a phase S
    constexpr int NA = NV;               // slots of a phase A
    constexpr int HALVES = 8;            // a chunk's probabilities come in 8 half units (one probability per lane each)
    static_assert(HALVES % NS == 0 && HALVES % (NS + NA) == 0, "phases divide the vector work evenly");
    static_assert(NS == NA, "one V block of A(0) is read per slot of S(0)");
    const char* kt = lds[2 * g + decltype(kb1)::value][0];
    const char* vt = lds[2 * g + decltype(vb0)::value][1];
    const float mc = m_run * c;
    bf16x8 kop[NK][2], vop[4][NV];
    float e[4][8];
    union {
      bf16x8 v;
      bf16x2 h[4];
    } pb[4];
    auto load_k = [&](int ks, int cb) {
      kop[ks][cb] = *reinterpret_cast<const bf16x8*>(kt + cb * 32 * ROW_BYTES + k_off[ks]);
    };
    auto load_v = [&](int chunk, int dblk) {
      const char* base = vt + 16 * chunk * ROW_BYTES + v_off[dblk];
      VOperand t;
      t.s.lo = lds_read_tr16(reinterpret_cast<const bf16_t*>(base));
      t.s.hi = lds_read_tr16(reinterpret_cast<const bf16_t*>(base + 8 * ROW_BYTES));
      vop[chunk][dblk] = t.v;
    };
    // Half unit u (0..7) of chunk `chunk`: one probability per lane; the odd ones also pack a pair and add it to
    // the row sum.
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
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) kop[0][cb] = k0[cb];
    float mx = -INFINITY;
    auto s_slot = [&](int gch, int i, int halves_chunk, int& half) {  // slot i of phase S(gch)
      const int ks = gch * KPC + (i >> 1), cb = i & 1;
      s_out[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[ks][cb], qreg[ks], s_out[cb], 0, 0, 0);
      fence();
      if (gch == 0) {  // the rest of this phase's K operands, and the V operands of A(0)
        if (ks + 1 < KPC) load_k(ks + 1, cb);
        load_v(0, i);
      }
      if (gch < 3) load_k(ks + KPC, cb);
      const int n = gch == 0 ? HALVES / NS : HALVES / (NS + NA);
      for (int u = 0; u < n; ++u) p_half(halves_chunk, half++);
      fence();
    };
    int half = 0;
#pragma unroll
    for (int i = 0; i < NS; ++i) s_slot(0, i, 0, half);
#pragma unroll
    for (int gch = 0; gch < 4; ++gch) {
      half = 0;
#pragma unroll
      for (int d = 0; d < NA; ++d) {  // slot d of phase A(gch)
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[gch][d], pb[gch].v, o[d], 0, 0, 0);
        fence();
        if (gch < 3) {
          load_v(gch + 1, d);
#pragma unroll
          for (int u = 0; u < HALVES / (NS + NA); ++u) p_half(gch + 1, half++);
        } else {  // the new scores are complete: their maxima, 32 / NA registers per slot
#pragma unroll
          for (int r = d * (32 / NA); r < (d + 1) * (32 / NA); ++r) mx = fmaxf(mx, s_out[r >> 4][r & 15]);
          asm volatile("" : "+v"(mx));  // keeps the partial maximum in this slot (it is only consumed on one branch later)
        }
        fence();
      }
      if (gch < 3) {
#pragma unroll
        for (int i = 0; i < NS; ++i) s_slot(gch + 1, i, gch + 1, half);
      }
    }
    return mx;
  };
  // The K operands of a step's first two MFMAs: read right after the barrier, before the step's tile copies are
  // issued, so that their LDS round trip passes under the scalar work of issuing.  Only those: right after a
  // barrier all wavefronts of the workgroup read at once, and what they ask for queues up in front of the first
  // MFMA; everything else is read from the slots of phase S(0) on.
  auto preload = [&](bf16x8 (&k0)[2], auto kb1) {
    const char* kt = lds[2 * g + decltype(kb1)::value][0];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) k0[cb] = *reinterpret_cast<const bf16x8*>(kt + cb * 32 * ROW_BYTES + k_off[0]);
  };

  f32x16 s_cur[2], s_nxt[2];
  // A wavefront whose 32 query rows all lie past t_k (ragged last query tile) keeps loading its share of
  // every tile and keeps the barriers, but leaves the matrix cores to the other workgroup on the unit.
  const bool active = q_row0 < t_k;
  // Steady-state step j (j + 1 < steps_all): K of the stream's tile j+1 sits in K stage kb1, V of its tile j in
  // V stage vb0.  s_in holds the scores of tile j, s_out receives those of tile j+1: the two register sets swap
  // roles from step to step instead of being copied.
  auto pipe_step = [&](int j, auto kb1, auto vb0, f32x16 (&s_in)[2], f32x16 (&s_out)[2]) {
    wait_vmcnt<0>();
    __syncthreads();
    if constexpr (FP8) {
      // What this step reads and arrived as codes: K(j+1), fetched during step j-1 into the K landing buffer, and
      // V(j) likewise.  Their stages are free (last read in step j-2), the landing buffers are free again after
      // the barrier, before this step's copies go out.
      const bool ck = j + 1 < tiles_all && j + 1 >= tiles_cur, cv = j >= tiles_cur;
      if (ck) tile::convert_raw8<false, 64 * NW>(raw_k, lds[decltype(kb1)::value][0], tid);
      if (cv) tile::convert_raw8<true, 64 * NW>(raw_v, lds[decltype(vb0)::value][1], tid);
      if (ck || cv) __syncthreads();
    }
    if constexpr (KS == 2) {  // two streams: the compiler's own order (a stream's last step may lack a successor tile)
      if (j + 2 < steps_all && has_tile(j + 2)) issue_k(j + 2, decltype(vb0)::value);
      if (has_tile(j + 1)) issue_v(j + 1, decltype(kb1)::value);
      if (!active) return;
      if (has_tile(j + 1)) scores(s_out, kb1);
      accumulate(s_in, vb0);
      if (has_tile(j + 1)) settle(j + 1, s_out);
      return;
    }
    bf16x8 k0[2];
    if (active) preload(k0, kb1);
    if (j + 2 < steps_all) issue_k(j + 2, decltype(vb0)::value);  // K stage j & 1: read by step j-1
    if (j > 0) issue_v(j + 1, decltype(kb1)::value);  // V stage (j+1) & 1 likewise; the prologue has already fetched V(1)
    if (!active) return;
    const float mx = step_math(s_in, s_out, k0, kb1, vb0);
    raise(mask_tail(j + 1, s_out) ? lane_max(s_out) : mx);
  };

  // Prologue: all four tile stages are free, so K(0), V(0), K(1) and V(1) all go out at once: one memory round
  // trip before the loop, and a walk of two tiles (every scale of up to 64 tokens) never waits for memory again.
  // Loads return in issue order, so waiting until only the copies younger than K(0) are outstanding means that
  // K(0) has landed (CPT copies per wavefront and bf16 tile, two per 8-bit tile); tile 0 is a current-scale tile,
  // whose address does not depend on the head's run.
  constexpr int CPT = TILE_BYTES / (1024 * NW);
  if (KS == 1) {
    issue_k(0, 0);
    issue_v(0, 0);
    if (tiles_all > 1) {
      issue_k(1, 1);
      issue_v(1, 1);
      if (FP8 && tiles_cur == 1)  // tile 1 arrives as codes: 8 / NW copies per wavefront for each of K(1), V(1)
        wait_vmcnt<CPT + 2 * (8 / NW)>();
      else
        wait_vmcnt<3 * CPT>();
    } else {
      wait_vmcnt<CPT>();
    }
  } else {  // a stream may have no tile at all, or one: everything it has goes out, then a full wait
    if (has_tile(0)) issue_k(0, 0);
    if (steps_all > 1 && has_tile(1)) issue_k(1, 1);
    if (has_tile(0)) issue_v(0, 0);
    wait_vmcnt<0>();
  }
  __syncthreads();
  if (active && has_tile(0)) {
    scores(s_cur, std::integral_constant<int, 0>{});
    settle(0, s_cur);
  }
  // Every path reaches the loop through a full wait that the compiler sees (a wavefront that skipped the scores
  // above never waited for its query rows): otherwise it waits for them inside every step, and with them for the
  // tile copies that the step has just issued.  The first step starts with the same wait, so this one is free.
  wait_vmcnt<0>();
  int it = 0;
  for (; it + 2 < steps_all; it += 2) {  // scores of even steps live in s_cur, of odd steps in s_nxt
    pipe_step(it, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{}, s_cur, s_nxt);
    pipe_step(it + 1, std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}, s_nxt, s_cur);
  }
  if (it + 1 < steps_all) {
    pipe_step(it, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{}, s_cur, s_nxt);
    ++it;
  }
  // Epilogue: the last tile has scores but no successor.
  wait_vmcnt<0>();
  __syncthreads();
  if constexpr (FP8) {
    if (it >= tiles_cur) {  // V of the last tile is still in its landing buffer
      if (it & 1)
        tile::convert_raw8<true, 64 * NW>(raw_v, lds[1][1], tid);
      else
        tile::convert_raw8<true, 64 * NW>(raw_v, lds[0][1], tid);
      __syncthreads();
    }
  }
  if (KS == 1 && QS == 1 && !active) return;
  if (active && has_tile(it)) {
    if (it & 1)
      accumulate(s_nxt, std::integral_constant<int, 1>{});
    else
      accumulate(s_cur, std::integral_constant<int, 0>{});
  }
  if constexpr (QS == 2) {  // the eight output tiles are staged over all four tile buffers: the V tiles must be done with
    __syncthreads();
    if (!active) return;
  }
  if constexpr (KS == 2) {
    // Stream 1 parks its accumulators (64 registers, one 256-byte row of LDS per register), row-sum partials and
    // references in the idle tile stages (66 KB from byte 48 K on: clear of the 16 KB at 0 and at 32 K where
    // stream 0 stages its output); stream 0 brings both halves to the larger reference and adds.
    __syncthreads();  // every wavefront has finished reading the tile stages
    float* park = reinterpret_cast<float*>(lds[1][1]) + wave * (66 * 64);
    if (g == 1 && active) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) park[(16 * i + r) * 64 + lane] = o[i][r];
      park[64 * 64 + lane] = m_run;
      park[65 * 64 + lane] = l_run;
    }
    __syncthreads();
    if (g == 1 || !active) return;
    const float m_other = park[64 * 64 + lane], l_other = park[65 * 64 + lane];
    const float m_new = fmaxf(m_run, m_other);  // m_run is finite: stream 0 always has tile 0
    const float a0 = fast_exp2((m_run - m_new) * c), a1 = fast_exp2((m_other - m_new) * c);  // 2^-inf = 0: no tile
    l_run = l_run * a0 + l_other * a1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] = o[i][r] * a0 + park[(16 * i + r) * 64 + lane] * a1;
  }

  const float l_tot = sum_halves(l_run);
  const float inv = 1.f / l_tot;
  // Output through LDS.  A lane owns one query row but only 4 consecutive columns at a time, so direct stores
  // would be 8-byte pieces scattered over 32 rows.  The K buffers are idle by now (their last reader passed the
  // barrier above and no copy is in flight), so every wavefront stages its 32 x d tile in half a K stage, with the
  // 16-byte chunks XORed with the row number, and writes it out as whole rows, 1 KB per instruction.
  char* stage = QS == 1 ? lds[wave >> 1][0] + (wave & 1) * (32 * ROW_BYTES)
                        : reinterpret_cast<char*>(lds) + wave_all * (32 * ROW_BYTES);
  // The lane numbers used from here on are formed anew from the work-item id, hidden from the optimiser, so that
  // they are not kept in registers (or spilled) across the tile loop, which has none to spare.
  int tid_o = threadIdx.x;
  asm volatile("" : "+v"(tid_o));
  const int lane_o = tid_o & 63, n_o = lane_o & 31, hl_o = lane_o >> 5;
#pragma unroll
  for (int dblk = 0; dblk < NV; ++dblk)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = static_cast<bf16_t>(o[dblk][4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(stage + n_o * ROW_BYTES + (((4 * dblk + g) ^ (n_o & (CPR - 1))) << 4) + 8 * hl_o) = v;
    }
  const int out_row0 = q_row0;
  bf16_t* op = static_cast<bf16_t*>(p.out) + cur_off + static_cast<long long>(out_row0) * D;
  constexpr int ROWS_PER_STORE = 64 / CPR;  // CPR lanes write one row
#pragma unroll
  for (int r = 0; r < 32 / ROWS_PER_STORE; ++r) {
    const int row = ROWS_PER_STORE * r + lane_o / CPR, slot = lane_o & (CPR - 1);
    const uint4 v = *reinterpret_cast<const uint4*>(stage + row * ROW_BYTES + ((slot ^ (row & (CPR - 1))) << 4));
    if (out_row0 + row < t_k) *reinterpret_cast<uint4*>(op + row * D + slot * 8) = v;
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

  if (static_cast<int>(blockIdx.x) >= p.attend_blocks) {  // fused append: a plain row copy
    const int j = blockIdx.x - p.attend_blocks;
    copy_rows_block(p.copy, j % p.ndesc, j / p.ndesc);
    return;
  }
  const int tid = threadIdx.x, r = tid >> 4, g = tid & 15;
  int id = blockIdx.x;
  const int qt = id % p.n_qtiles;
  id /= p.n_qtiles;
  const int b = id % p.batch;
  const HeadWork hw = p.work[id / p.batch];
  const int h = hw.head;

  const int t_k = p.t_k;
  const int n_prior = hw.run_len;
  const int n_total = n_prior + t_k;
  const long long cur_off = (static_cast<long long>(b) * p.H + h) * t_k * D;
  const long long run_off = (static_cast<long long>(b) * p.arena_tokens + hw.run_row) * D;
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

namespace {

constexpr int TWO_STREAM_LDS_BYTES = 2 * 2 * 2 * TILE_BYTES_D128;  // two streams x two stages x (K, V)
constexpr int FP8_LDS_BYTES = 2 * 2 * TILE_BYTES_D128 + 2 * tile::RAW8_BYTES;  // two stages x (K, V) + two landing buffers
constexpr int TWO_STREAM_MAX_BLOCKS = 256;                    // compute units of the chip
constexpr int TWO_STREAM_MIN_TOKENS = 384;                    // shorter walks gain nothing (measured at 256)
// Two query sets per workgroup: from this scale size on, when the launch still gives every compute unit two rounds
// of such workgroups (measured: a single round of 256 is slower than 512 workgroups of 128 queries), and when the
// last 256-query tile is not mostly empty (1600 tokens: 7 tiles, the last one a quarter full, measured slower).
constexpr int TWO_SET_MIN_TOKENS = 1024;
constexpr int TWO_SET_MIN_BLOCKS = 512;

// 128 KB of dynamic LDS need the function attribute raised, once per device.
hipError_t allow_two_stream_lds() {
  static std::atomic<unsigned long long> done{0};  // one bit per device ordinal below 64
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && (done.load(std::memory_order_acquire) >> dev & 1)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_bf16_kernel<2, false, 128>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, TWO_STREAM_LDS_BYTES);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_bf16_kernel<1, true, 128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FP8_LDS_BYTES);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_bf16_kernel<1, true, 128, 2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, FP8_LDS_BYTES);
  if (e == hipSuccess && dev >= 0 && dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
  return e;
}

}  // namespace

hipError_t attend_prepare_device() { return allow_two_stream_lds(); }

hipError_t launch_attend(const AttendArgs& a, hipStream_t stream) {
  AttendParams p{};
  p.H = a.H;
  p.batch = a.batch;
  p.t_k = a.t_k;
  p.arena_tokens = a.arena_tokens;
  p.work = a.work;
  p.uniform_len = a.uniform_len;
  p.uniform_row0 = a.uniform_row0;
  p.q = a.q;
  p.k_cur = a.k_cur;
  p.v_cur = a.v_cur;
  p.k_arena = a.k_arena;
  p.v_arena = a.v_arena;
  p.out = a.out;
  p.sm_scale = a.sm_scale;
  p.ndesc = a.ndesc;
  unsigned copy_blocks = 0;
  if (a.ndesc > 0) {
    if (a.row_bytes % 16 != 0) return hipErrorInvalidValue;
    p.copy.chunks_per_row = a.row_bytes / 16;
    p.copy.kv_fp8 = a.kv_fp8 ? 1 : 0;
    p.copy.H = a.H;
    p.copy.t_k = a.t_k;
    p.copy.arena_tokens = a.arena_tokens;
    p.copy.descs = a.descs;
    p.copy.k_new = static_cast<const uint4*>(a.k_cur);
    p.copy.v_new = static_cast<const uint4*>(a.v_cur);
    p.copy.k_arena = static_cast<uint4*>(a.k_arena_rw);
    p.copy.v_arena = static_cast<uint4*>(a.v_arena_rw);
    copy_blocks = unsigned(a.ndesc) * a.batch;
  }
  if (a.dtype == HEATKV_BF16) {
    if (a.d != 128 && a.d != 64) return hipErrorInvalidValue;
    if (a.d == 64 && a.kv_fp8) return hipErrorInvalidValue;
    p.n_qtiles = (a.t_k + BM - 1) / BM;
    const unsigned pairs8 = (unsigned(a.H) * a.batch + 7) / 8 * 8;  // padded so that id % 8 is the XCD
    p.attend_blocks = int(unsigned(p.n_qtiles) * pairs8);
    const dim3 grid(unsigned(p.attend_blocks) + copy_blocks);
    // Long walks on a full chip: 256 queries per workgroup share every K/V tile (d = 128, either cache format).
    const int wide = (a.t_k + 2 * BM - 1) / (2 * BM);
    const bool two_sets = a.d == 128 && a.t_k >= TWO_SET_MIN_TOKENS &&
                          unsigned(wide) * pairs8 >= unsigned(TWO_SET_MIN_BLOCKS) && (wide * 2 * BM - a.t_k) * 16 <= a.t_k;
    const unsigned wide_blocks = unsigned(wide) * pairs8;
    if (a.d == 64) {  // rows of 128 bytes: the single-stream instance
      hipLaunchKernelGGL((attend_bf16_kernel<1, false, 64>), grid, dim3(256), 0, stream, p);
    } else if (a.kv_fp8) {  // 8-bit cache rows: the single-stream instances with landing buffers
      const hipError_t e = allow_two_stream_lds();
      if (e != hipSuccess) return e;
      if (two_sets) {
        p.n_qtiles = wide;
        p.attend_blocks = int(wide_blocks);
        hipLaunchKernelGGL((attend_bf16_kernel<1, true, 128, 2>), dim3(wide_blocks + copy_blocks), dim3(512),
                           FP8_LDS_BYTES, stream, p);
      } else {
        hipLaunchKernelGGL((attend_bf16_kernel<1, true, 128>), grid, dim3(256), FP8_LDS_BYTES, stream, p);
      }
    } else if (p.attend_blocks <= TWO_STREAM_MAX_BLOCKS && a.t_k >= TWO_STREAM_MIN_TOKENS) {
      // At most one workgroup per compute unit: two key streams per workgroup put two wavefronts on every SIMD.
      const hipError_t e = allow_two_stream_lds();
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL((attend_bf16_kernel<2, false, 128>), grid, dim3(512), TWO_STREAM_LDS_BYTES, stream, p);
    } else if (two_sets) {
      p.n_qtiles = wide;
      p.attend_blocks = int(wide_blocks);
      hipLaunchKernelGGL((attend_bf16_kernel<1, false, 128, 2>), dim3(wide_blocks + copy_blocks), dim3(512), 0, stream, p);
    } else {
      hipLaunchKernelGGL((attend_bf16_kernel<1, false, 128>), grid, dim3(256), 0, stream, p);
    }
  } else {
    if (a.kv_fp8) return hipErrorInvalidValue;
    p.n_qtiles = (a.t_k + FQ - 1) / FQ;
    p.attend_blocks = int(unsigned(p.n_qtiles) * a.H * a.batch);
    const dim3 grid(unsigned(p.attend_blocks) + copy_blocks);
    if (a.d == 64)
      hipLaunchKernelGGL(attend_f32_kernel<64>, grid, dim3(256), 0, stream, p);
    else if (a.d == 128)
      hipLaunchKernelGGL(attend_f32_kernel<128>, grid, dim3(256), 0, stream, p);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace heatkv

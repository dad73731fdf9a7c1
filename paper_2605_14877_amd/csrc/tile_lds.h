// The LDS tile format shared by the bf16 kernels (attention, calibration, the measurement probes): how a 64-row
// K or V tile travels from HBM into LDS and where the matrix-core operand reads find their data in it.
//
// A tile is 64 rows of 256 bytes (d = 128 bf16) or 128 bytes (d = 64), row-major, unpadded.  The 16-byte chunks of a
// row are XOR-swizzled with the row number; the lane that fills an LDS slot simply fetches the matching global chunk,
// so the swizzle costs nothing on the way in.  Copies are global_load_lds_dwordx4 (HBM -> LDS without
// registers): each of a workgroup's four wavefronts issues four (two) of them per tile, 1 KB each.
#pragma once

#include "device_util.h"

namespace heatkv {
namespace tile {

constexpr int ROWS = 64;            // keys per tile
constexpr int ROW_BYTES = 256;      // one bf16 row of 128 elements (the default row size RB below)
constexpr int BYTES = ROWS * ROW_BYTES;

// Everything below takes the row size RB in bytes as a template parameter: 256 (d = 128) or 128 (d = 64).  A tile
// is ROWS x RB bytes; a row holds RB / 16 chunks.

// The LDS has 64 four-byte banks (256 bytes per clock).
// K tiles: ds_read_b128 serves 16 consecutive lanes per clock; they read the same logical chunk of 16
// consecutive rows.  256-byte rows all start on bank 0, so the chunk is XORed with row % 16 and the 16 accesses
// cover all 64 banks (measured 246 bytes/clock per compute unit against 128 with an 8-row pattern).  128-byte rows
// alternate between the two halves of the bank space, so XORing the chunk (3 bits) with (row / 2) % 8 does the same.
// V tiles: the transposing 8-byte read serves 32 lanes per clock, a block of 4 rows x 64 bytes; XORing the
// 64-byte window index with row % 4 (256-byte rows: chunk bits 2-3) or with (row / 2) % 2 (128-byte rows: chunk
// bit 2, the two rows of a pair already lie in different halves) puts the four rows on four different bank
// quarters (measured 156-162 bytes/clock, the instruction's ceiling, against 125).
// All of them depend only on row % 16, so they are the same for the rows a lane loads in one tile (16 or 32 apart).
template <int RB = ROW_BYTES>
__device__ __forceinline__ int swizzle_k(int row) {
  static_assert(RB == 256 || RB == 128, "row of 128 or 64 bf16 elements");
  return RB == 256 ? (row & 15) : ((row >> 1) & 7);
}
template <int RB = ROW_BYTES>
__device__ __forceinline__ int swizzle_v(int row) {
  return RB == 256 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

// Loader geometry.  A wavefront copies 1 KB per instruction: wavefront w fills LDS bytes [(4j + w) KB, +1 KB) of a
// tile with instruction j (four instructions for a 16 KB tile, two for an 8 KB one); lane L lands on byte 16 L of
// that range, i.e. row loader_row0 + (4096 / RB) j, slot L % (RB / 16).  The swizzle is the same for all j, so one
// per-lane offset serves all instructions (the 4 KB step between them goes into the scalar base addresses).
template <int RB = ROW_BYTES>
__device__ __forceinline__ int loader_row0(int wave, int lane) {
  return RB == 256 ? 4 * wave + (lane >> 4) : 8 * wave + (lane >> 3);
}
template <int RB = ROW_BYTES>
__device__ __forceinline__ int loader_off_k(int wave, int lane) {
  const int r = loader_row0<RB>(wave, lane);
  return r * RB + (((lane & (RB / 16 - 1)) ^ swizzle_k<RB>(r)) << 4);
}
template <int RB = ROW_BYTES>
__device__ __forceinline__ int loader_off_v(int wave, int lane) {
  const int r = loader_row0<RB>(wave, lane);
  return r * RB + (((lane & (RB / 16 - 1)) ^ swizzle_v<RB>(r)) << 4);
}

// One 1 KB copy: 64 lanes x 16 bytes from src + lane_off (per-lane byte offset) to LDS byte address lds_dst +
// 16 * lane.  Raw instruction on purpose: when the compiler sees an LDS-writing load it orders every later LDS
// read after it (a full wait in the middle of the math); here the ordering is the caller's s_waitcnt vmcnt +
// workgroup barrier.  The instruction takes its LDS base from M0; the operand is bound to that register, so the
// compiler writes M0 itself and knows that it did.
// Two hazards that the compiler covers for its own instructions but not for text: an LDS-DMA instruction needs one
// wait state after a scalar write of M0, and a vector-memory instruction must not read a scalar register within
// five wait states of a vector-ALU write to it (v_readlane, which is how a spilled scalar comes back: seen for
// the source address when scalar registers ran short).  The leading s_mov_b64 settles both: it is the instruction
// between the M0 write and the copy, and the copy reads the address from the pair this scalar instruction wrote
// (scalar-ALU results need no wait states before a vector-memory read, and a scalar instruction reading a
// vector-written scalar register is interlocked by the hardware).
__device__ __forceinline__ void copy_1k(unsigned lds_dst, int lane_off, const char* src) {
  unsigned long long base;
  asm volatile("s_mov_b64 %0, %2\n\tglobal_load_lds_dwordx4 %1, %0"
               : "=&s"(base)
               : "v"(lane_off), "s"(src), "{m0}"(lds_dst)
               : "memory");
}
// The same instruction under another text, for the ragged-tile path: the differing text keeps the compiler from
// merging the two paths back into one statement with per-lane selected operands (24 vector instructions in
// every step of the common path).
__device__ __forceinline__ void copy_1k_ragged(unsigned lds_dst, int lane_off, const char* src) {
  unsigned long long base;
  asm volatile("s_mov_b64 %0, %2\n\tglobal_load_lds_dwordx4 %1, %0\n\t; ragged"
               : "=&s"(base)
               : "v"(lane_off), "s"(src), "{m0}"(lds_dst)
               : "memory");
}

// This wavefront's copies of a full tile: `src` = first byte of the tile's 64 contiguous rows, `lds_tile` =
// LDS byte address of the tile, lane_off = loader_off_k / loader_off_v.  NW wavefronts (`wave` = 0..NW-1) share a
// tile: each copies ROWS * RB / (1024 NW) KB of it, instruction j covering the KB at (NW j + wave).
template <int RB = ROW_BYTES, int NW = 4>
__device__ __forceinline__ void issue_full(unsigned lds_tile, int wave, int lane_off, const char* src) {
#pragma unroll
  for (int j = 0; j < ROWS * RB / (1024 * NW); ++j)
    copy_1k(lds_tile + wave * 1024 + j * (1024 * NW), lane_off, src + j * (1024 * NW));
}
// The same for a tile with only `left` (1..63) valid rows: rows past the end re-read the last valid row (the
// caller masks their scores).  SWZ_V selects the V swizzle.
template <bool SWZ_V, int RB = ROW_BYTES, int NW = 4>
__device__ __forceinline__ void issue_ragged(unsigned lds_tile, int wave, int lane, int left, const char* src) {
  const int row0 = loader_row0<RB>(wave, lane);
#pragma unroll
  for (int j = 0; j < ROWS * RB / (1024 * NW); ++j) {
    const int row = row0 + (1024 * NW / RB) * j;
    const int rr = row < left ? row : left - 1;
    const int off = rr * RB + (((lane & (RB / 16 - 1)) ^ (SWZ_V ? swizzle_v<RB>(row) : swizzle_k<RB>(row))) << 4);
    copy_1k_ragged(lds_tile + wave * 1024 + j * (1024 * NW), off, src);
  }
}

// 8-bit cache rows (FP8 E4M3 codes, 128 bytes per row): a 64-row tile is 8 KB and lands in LDS as it lies in
// memory, 8 / NW KB per wavefront (NW wavefronts share a tile) in copies of 1 KB; `left` < 64: rows past the end
// re-read the last valid row.
constexpr int RAW8_ROW_BYTES = 128;
constexpr int RAW8_BYTES = ROWS * RAW8_ROW_BYTES;
template <int NW = 4>
__device__ __forceinline__ void issue_raw8(unsigned lds_tile, int wave, int lane, int left, const char* src) {
  constexpr int PER_WAVE = RAW8_BYTES / NW;  // bytes of the tile this wavefront copies
  if (left >= ROWS) {
#pragma unroll
    for (int j = 0; j < PER_WAVE / 1024; ++j)
      copy_1k(lds_tile + wave * PER_WAVE + j * 1024, lane * 16, src + wave * PER_WAVE + j * 1024);
  } else {
#pragma unroll
    for (int j = 0; j < PER_WAVE / 1024; ++j) {
      const int row = (ROWS / NW) * wave + 8 * j + (lane >> 3);
      const int rr = row < left ? row : left - 1;
      copy_1k_ragged(lds_tile + wave * PER_WAVE + j * 1024, rr * RAW8_ROW_BYTES + (lane & 7) * 16, src);
    }
  }
}
// Turns a landed 8-bit tile (`raw`, LDS) into the bf16 tile format at `stage` (LDS): NT lanes, 1024 / NT groups of
// eight codes each; every E4M3 value is a bf16 value, so the conversion is exact.  SWZ_V selects the V swizzle.
template <bool SWZ_V, int NT = 256>
__device__ __forceinline__ void convert_raw8(const char* raw, char* stage, int tid) {
  // The per-lane offsets below are cheap; made opaque here so that they are recomputed on the spot instead of being
  // kept in registers across the caller's tile loop, which has none to spare.
  asm volatile("" : "+v"(tid));
#pragma unroll
  for (int i = 0; i < 1024 / NT; ++i) {
    const int idx = tid + NT * i;
    const int row = idx >> 4, lc = idx & 15;
    const uint2 w = *reinterpret_cast<const uint2*>(raw + row * RAW8_ROW_BYTES + lc * 8);
    union {
      bf16x2 h[4];
      uint4 u;
    } o;
    o.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w.x), 1.0f, false);
    o.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w.x), 1.0f, true);
    o.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w.y), 1.0f, false);
    o.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(static_cast<int>(w.y), 1.0f, true);
    const int pc = lc ^ (SWZ_V ? swizzle_v(row) : swizzle_k(row));
    *reinterpret_cast<uint4*>(stage + row * ROW_BYTES + (pc << 4)) = o.u;
  }
}

// Reader offsets inside a tile for the 32x32x16 MFMA operand layouts (lane = n + 32 hl, n = lane % 32); NK = d / 16
// and NV = d / 32 entries.
// K as the A operand of S^T = K Q^T: row n (+32 per column block), chunk 2 ks + hl for ks = 0..NK-1.
template <int RB = ROW_BYTES>
__device__ __forceinline__ void reader_off_k(int lane, int (&k_off)[RB / 32]) {
  const int n = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < RB / 32; ++ks) k_off[ks] = n * RB + (((2 * ks + hl) ^ swizzle_k<RB>(n)) << 4);
}
// V^T as the A operand of O^T += V^T P^T through the transposing read: lane i of a 16-lane group points at row
// key0 + 4 hl + i / 4, columns 32 dblk + 16 (group & 1) + 4 (i % 4) .. +3, and receives column i of that 4 x 16 block.
template <int RB = ROW_BYTES>
__device__ __forceinline__ void reader_off_v(int lane, int (&v_off)[RB / 64]) {
  const int hl = lane >> 5, tr_i = lane & 15, tr_grp = lane >> 4;
  const int v_row = 4 * hl + (tr_i >> 2);
#pragma unroll
  for (int dblk = 0; dblk < RB / 64; ++dblk) {
    const int chunk = 4 * dblk + 2 * (tr_grp & 1) + ((tr_i & 3) >> 1);
    v_off[dblk] = v_row * RB + ((chunk ^ swizzle_v<RB>(v_row)) << 4) + ((tr_i & 1) << 3);
  }
}

}  // namespace tile
}  // namespace heatkv

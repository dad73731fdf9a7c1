// The LDS tile format shared by the bf16 kernels (attention, calibration, the measurement probes): how a 64-row
// K or V tile travels from HBM into LDS and where the matrix-core operand reads find their data in it.
//
// A tile is 64 rows of 256 bytes (d = 128 bf16), row-major, unpadded.  The sixteen 16-byte chunks of a row are
// XOR-swizzled with the row number; the lane that fills an LDS slot simply fetches the matching global chunk,
// so the swizzle costs nothing on the way in.  Copies are global_load_lds_dwordx4 (HBM -> LDS without
// registers): each of a workgroup's four wavefronts issues four of them per tile, 1 KB each.
#pragma once

#include "device_util.h"

namespace heatkv {
namespace tile {

constexpr int ROWS = 64;            // keys per tile
constexpr int ROW_BYTES = 256;      // one bf16 row of 128 elements
constexpr int BYTES = ROWS * ROW_BYTES;

// The LDS has 64 four-byte banks (256 bytes per clock).
// K tiles: ds_read_b128 serves 16 consecutive lanes per clock; they read the same logical chunk of 16
// consecutive rows, so the chunk is XORed with row % 16 and the 16 accesses cover all 64 banks (measured
// 246 bytes/clock per compute unit against 128 with an 8-row pattern).
// V tiles: the transposing 8-byte read serves 32 lanes per clock, a block of 4 rows x 64 bytes; XORing the
// 64-byte window index (chunk bits 2-3) with row % 4 puts the four rows on four different bank quarters
// (measured 156-162 bytes/clock, the instruction's ceiling, against 125).
// Both depend only on row % 16, so they are the same for the four rows a lane loads in one tile (16 apart).
__device__ __forceinline__ int swizzle_k(int row) { return row & 15; }
__device__ __forceinline__ int swizzle_v(int row) { return (row & 3) << 2; }

// Loader geometry.  Wavefront w fills LDS bytes [(4j + w) KB, +1 KB) of a tile with instruction j = 0..3;
// lane L lands on byte 16 L of that range, i.e. row loader_row0 + 16 j, slot L % 16.  The swizzle is the same
// for all j, so one per-lane offset serves the four instructions (the 4 KB step between them goes into the
// scalar base addresses).
__device__ __forceinline__ int loader_row0(int wave, int lane) { return 4 * wave + (lane >> 4); }
__device__ __forceinline__ int loader_off_k(int wave, int lane) {
  const int r = loader_row0(wave, lane);
  return r * ROW_BYTES + (((lane & 15) ^ swizzle_k(r)) << 4);
}
__device__ __forceinline__ int loader_off_v(int wave, int lane) {
  const int r = loader_row0(wave, lane);
  return r * ROW_BYTES + (((lane & 15) ^ swizzle_v(r)) << 4);
}

// One 1 KB copy: 64 lanes x 16 bytes from src + lane_off (per-lane byte offset) to LDS byte address lds_dst +
// 16 * lane.  Raw instruction on purpose: when the compiler sees an LDS-writing load it orders every later LDS
// read after it (a full wait in the middle of the math); here the ordering is the caller's s_waitcnt vmcnt +
// workgroup barrier.  The instruction takes its LDS base from M0; the operand is bound to that register, so the
// compiler writes M0 itself and knows that it did.  The leading s_nop is the wait state between a scalar write of
// M0 and an LDS-DMA instruction that reads it (the compiler inserts it for its own such loads, not for text).
__device__ __forceinline__ void copy_1k(unsigned lds_dst, int lane_off, const char* src) {
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(src), "{m0}"(lds_dst) : "memory");
}
// The same instruction under another text, for the ragged-tile path: the differing text keeps the compiler from
// merging the two paths back into one statement with per-lane selected operands (24 vector instructions in
// every step of the common path).
__device__ __forceinline__ void copy_1k_ragged(unsigned lds_dst, int lane_off, const char* src) {
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\t; ragged" ::"v"(lane_off), "s"(src), "{m0}"(lds_dst) : "memory");
}

// This wavefront's four copies of a full tile: `src` = first byte of the tile's 64 contiguous rows, `lds_tile` =
// LDS byte address of the tile, lane_off = loader_off_k / loader_off_v.
__device__ __forceinline__ void issue_full(unsigned lds_tile, int wave, int lane_off, const char* src) {
#pragma unroll
  for (int j = 0; j < 4; ++j) copy_1k(lds_tile + wave * 1024 + j * 4096, lane_off, src + j * (16 * ROW_BYTES));
}
// The same for a tile with only `left` (1..63) valid rows: rows past the end re-read the last valid row (the
// caller masks their scores).  SWZ_V selects the V swizzle.
template <bool SWZ_V>
__device__ __forceinline__ void issue_ragged(unsigned lds_tile, int wave, int lane, int left, const char* src) {
  const int row0 = loader_row0(wave, lane);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = row0 + 16 * j;
    const int rr = row < left ? row : left - 1;
    const int off = rr * ROW_BYTES + (((lane & 15) ^ (SWZ_V ? swizzle_v(row) : swizzle_k(row))) << 4);
    copy_1k_ragged(lds_tile + wave * 1024 + j * 4096, off, src);
  }
}

// 8-bit cache rows (FP8 E4M3 codes, 128 bytes per row): a 64-row tile is 8 KB and lands in LDS as it lies in
// memory, 2 KB per wavefront in two copies; `left` < 64: rows past the end re-read the last valid row.
constexpr int RAW8_ROW_BYTES = 128;
constexpr int RAW8_BYTES = ROWS * RAW8_ROW_BYTES;
__device__ __forceinline__ void issue_raw8(unsigned lds_tile, int wave, int lane, int left, const char* src) {
  if (left >= ROWS) {
#pragma unroll
    for (int j = 0; j < 2; ++j) copy_1k(lds_tile + wave * 2048 + j * 1024, lane * 16, src + wave * 2048 + j * 1024);
  } else {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = 16 * wave + 8 * j + (lane >> 3);
      const int rr = row < left ? row : left - 1;
      copy_1k_ragged(lds_tile + wave * 2048 + j * 1024, rr * RAW8_ROW_BYTES + (lane & 7) * 16, src);
    }
  }
}
// Turns a landed 8-bit tile (`raw`, LDS) into the bf16 tile format at `stage` (LDS): 256 lanes, four groups of
// eight codes each; every E4M3 value is a bf16 value, so the conversion is exact.  SWZ_V selects the V swizzle.
template <bool SWZ_V>
__device__ __forceinline__ void convert_raw8(const char* raw, char* stage, int tid) {
  // The per-lane offsets below are cheap; made opaque here so that they are recomputed on the spot instead of being
  // kept in registers across the caller's tile loop, which has none to spare.
  asm volatile("" : "+v"(tid));
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int idx = tid + 256 * i;
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

// Reader offsets inside a tile for the 32x32x16 MFMA operand layouts (lane = n + 32 hl, n = lane % 32).
// K as the A operand of S^T = K Q^T: row n (+32 per column block), chunk 2 ks + hl for ks = 0..7.
__device__ __forceinline__ void reader_off_k(int lane, int (&k_off)[8]) {
  const int n = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_off[ks] = n * ROW_BYTES + (((2 * ks + hl) ^ swizzle_k(n)) << 4);
}
// V^T as the A operand of O^T += V^T P^T through the transposing read: lane i of a 16-lane group points at row
// key0 + 4 hl + i / 4, columns 32 dblk + 16 (group & 1) + 4 (i % 4) .. +3, and receives column i of that 4 x 16 block.
__device__ __forceinline__ void reader_off_v(int lane, int (&v_off)[4]) {
  const int hl = lane >> 5, tr_i = lane & 15, tr_grp = lane >> 4;
  const int v_row = 4 * hl + (tr_i >> 2);
#pragma unroll
  for (int dblk = 0; dblk < 4; ++dblk) {
    const int chunk = 4 * dblk + 2 * (tr_grp & 1) + ((tr_i & 3) >> 1);
    v_off[dblk] = v_row * ROW_BYTES + ((chunk ^ swizzle_v(v_row)) << 4) + ((tr_i & 1) << 3);
  }
}

}  // namespace tile
}  // namespace heatkv

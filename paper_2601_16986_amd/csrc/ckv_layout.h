// Tiled K/V layout of one unit's cache, shared by host (import/export) and
// device code of the library.
//
// Entries are grouped in blocks of 32; one block of K (or V) is 32 x 128 bf16
// = 8 KB, stored as 8 chunks of 1 KB.  A 64-lane wavefront reads one chunk with
// one 16-byte load per lane (lane l takes bytes [16 l, 16 l + 16)), and the 8
// bf16 a lane receives are exactly its operand elements of a
// v_mfma_f32_16x16x32_bf16:
//
//  K block, chunk (tt, s), tt = 0..1 (entries 16 tt .. 16 tt + 15),
//                          s  = 0..3 (dims 32 s .. 32 s + 31):
//     lane (j = l % 16, kg = l / 16) holds K[entry 16 tt + j][dims 32 s + 8 kg + e], e = 0..7
//     -> A operand (rows = entries, k = dims) of the QK^T product.
//
//  V block, chunk dt = 0..7 (dims 16 dt .. 16 dt + 15):
//     lane (j, kg) holds V[entry ent(kg, e)][dim 16 dt + j], e = 0..7, with
//     ent(kg, e) = 4 kg + e for e < 4 and 16 + 4 kg + (e - 4) otherwise
//     -> B operand (k = entries, cols = dims) of the PV product; the entry
//     order matches the lane layout in which QK^T leaves the logits, so the
//     probabilities feed the second MFMA without any cross-lane movement.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define CKV_HD __host__ __device__ __forceinline__
#else
#define CKV_HD inline
#endif

namespace ckv {

constexpr int kDim = 128;          // head_dim
constexpr int kBlk = 32;           // entries per block
constexpr int kBlkElems = kBlk * kDim;   // bf16 elements per block (4096)
constexpr int kChunkBlocks = 8;    // blocks per scan work item
constexpr int kChunk = kBlk * kChunkBlocks;   // 256 entries
constexpr int kMaxGroup = 8;       // query heads per KV head
constexpr int kSeg = kChunk;                // entries per segment, the unit in which pool memory is handed to units (64 KB of K, 64 KB of V)
constexpr int kSegBlocks = kChunkBlocks;
constexpr int kSegElems = kSeg * kDim;      // bf16 elements of one segment in the K (or V) pool

// element offset (in bf16) of K[entry r][dim c] from the start of the run of blocks that holds entry 0
// (a unit's entries are contiguous inside a segment of 256: callers pass r % 256 and add the segment's offset)
CKV_HD int64_t k_offset(int r, int c) {
  int blk = r >> 5, rr = r & 31;
  int tt = rr >> 4, j = rr & 15;
  int s = c >> 5, kg = (c & 31) >> 3, e = c & 7;
  return (int64_t)blk * kBlkElems + (((tt * 4 + s) * 64 + kg * 16 + j) << 3) + e;
}

// the same for V[entry r][dim c]
CKV_HD int64_t v_offset(int r, int c) {
  int blk = r >> 5, rr = r & 31;
  int tt = rr >> 4, kg = (rr & 15) >> 2, e = tt * 4 + (rr & 3);
  int dt = c >> 4, j = c & 15;
  return (int64_t)blk * kBlkElems + (((dt * 64) + kg * 16 + j) << 3) + e;
}

}  // namespace ckv

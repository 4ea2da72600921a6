// Internal: the plan blob shared by the host planner and the kernels.
//
// The blob is position independent (offsets, no pointers) so the caller can copy
// it to the device byte for byte.  It holds the result of Alg. 1's prefill loop
// (which chunk goes to which bitwidth class, in which order) plus the derived
// block layout of the packed cache and the static work split of the decode kernel.
#pragma once
#include <stdint.h>

namespace cocktail {

constexpr uint32_t kPlanMagic = 0x434b544cu;  // "CKTL"
constexpr uint32_t kPlanVersion = 8;
constexpr int kTB = 64;                        // tokens per block
constexpr int kNumClasses = 3;
constexpr int kPartialFloats = 2;              // (m, l) in front of the D output values

// One contiguous run of blocks of one (sequence, kv head, class).
struct Segment {
  int32_t b, h, cls, ntok;   // ntok: valid tokens of the whole run (last block may be partial)
  int32_t blk0;              // first block, index into the class buffer
  int32_t nblk;
  int32_t gblk0;             // first block in the global order (static part of every class, then dynamic part)
  int32_t bh;                // b * Hkv + h
};

// Everything a decode workgroup needs to start streaming, in one 64-byte record.
struct WorkerRec {
  int32_t g0, g1;            // global block range [g0, g1)
  int32_t seg0;              // index of the segment holding g0
  int32_t pid0;              // first partial id this worker writes
  Segment first;             // copy of segments[seg0]
  int32_t pad[4];
};
static_assert(sizeof(WorkerRec) == 64, "WorkerRec is one 64-byte line");

struct PlanHeader {
  uint32_t magic, version;
  int32_t batch, num_q_heads, num_kv_heads, head_dim, chunk_size, group_size;
  int32_t rep;               // Hq / Hkv
  int32_t num_workers, num_segments, num_partials;
  int32_t total_gblocks, pad0;
  int64_t total_chunks;
  int64_t total_tokens;
  int64_t class_blocks[kNumClasses];
  int64_t class_bytes[kNumClasses];
  int32_t block_bytes[kNumClasses];
  int32_t row_bytes[kNumClasses];     // code bytes per token row
  int64_t workspace_bytes;
  int64_t plan_bytes;
  int64_t packed_bytes;
  // byte offsets of the arrays inside the blob (each 16-byte aligned)
  int32_t off_seq_len;        // int32 [B]
  int32_t off_cum_tokens;     // int64 [B+1]
  int32_t off_chunk_off;      // int32 [B+1]   prefix of N_b
  int32_t off_perm;           // int32 [total_chunks]  per-sequence chunk indices, gather form
  int32_t off_class_tokens;   // int32 [B][3]
  int32_t off_class_chunk0;   // int32 [B][3]  first position in perm_b of class c
  int32_t off_blk_base;       // int32 [B+1][3] first block of sequence b in class buffer c
  int32_t off_nblk;           // int32 [B][3]  blocks per head
  int32_t off_segments;       // Segment [num_segments]
  int32_t off_bh_pid;         // int32 [B*Hkv][3][2][2] partial ids [begin, end) of each (b, kv head, class, part)
  int32_t off_worker_rec;     // WorkerRec [P + Q]: P static ranges, then the Q small items in dispatch order
  int32_t num_items;          // Q
  int32_t pad1[4];
};

template <typename T>
__host__ __device__ inline const T* plan_array(const void* blob, int32_t off) {
  return reinterpret_cast<const T*>(static_cast<const char*>(blob) + off);
}

}  // namespace cocktail

// Internal: the plan blob shared by the host planner and the kernels.
//
// The blob is position independent (offsets, no pointers) so the caller can copy
// it to the device byte for byte.  It holds the result of Alg. 1's prefill loop
// (which chunk goes to which bitwidth class, in which order) plus the derived
// block layout of the packed cache and the work split of the decode kernel.
#pragma once
#include <stdint.h>

namespace cocktail {

constexpr uint32_t kPlanMagic = 0x434b544cu;  // "CKTL"
constexpr uint32_t kPlanVersion = 15;
constexpr int kTB = 64;                        // tokens per block
constexpr int kNumClasses = 4;                 // INT2, INT4, INT8, FP16: the order of the concatenation
constexpr int kFp16Class = kNumClasses - 1;
constexpr int kClassBits[kNumClasses] = {2, 4, 8, 16};
constexpr int kPartialFloats = 4;              // (m, l, tokens covered as int32, unused) in front of the D output values
// Units one wave consumes per loop iteration in class INT2, INT4, INT8, FP16: the grain of the shared pools.
#ifndef COCKTAIL_J2
#define COCKTAIL_J2 4
#endif
#ifndef COCKTAIL_J4
#define COCKTAIL_J4 2
#endif
#ifndef COCKTAIL_J8
#define COCKTAIL_J8 1
#endif
#ifndef COCKTAIL_J16
#define COCKTAIL_J16 1
#endif
constexpr int kIterUnits[kNumClasses] = {COCKTAIL_J2, COCKTAIL_J4, COCKTAIL_J8, COCKTAIL_J16};
constexpr int kMaxPoolSegments = 32;           // segments one pool may touch (a worker tracks them in a bit mask)
// The appended tokens of a (sequence, kv head) are attended to by one extra workgroup per this many 64-token
// blocks of append capacity (one partial state each), so a long generation does not hang on a single wave.
constexpr int kAppendSliceBlocks = 8;
constexpr int kCounterStride = 32;             // uint32 slots between two pool counters (one 128-byte line each)
// Query heads per kv head for which a wave serves four of them at a time with matrix instructions and V is
// stored in token quads: 2 to 4 heads take one wave per workgroup, 5 to 8 two waves (one per head quad).
constexpr int kQuadMinRep = 2, kQuadMaxRep = 8;
__host__ __device__ inline bool uses_token_quads(int rep) { return rep >= kQuadMinRep && rep <= kQuadMaxRep; }
__host__ __device__ inline int quad_waves(int rep) { return (rep + 3) / 4; }
// Query heads one workgroup serves when rep = Hq / Hkv heads share a kv head: all of them up to kQuadMaxRep; beyond
// that the heads of a kv head are cut into equal sets (the largest divisor of rep that the matrix kernel takes),
// each walking the kv head's blocks by itself; 1 (a wave per query head, vector ALU) if there is no such divisor
// or the plan asks for it.
__host__ __device__ inline int work_rep_of(int rep, bool vector_alu_only) {
  if (vector_alu_only || rep <= 1) return 1;
  if (rep <= kQuadMaxRep) return rep;
  for (int d = kQuadMaxRep; d >= kQuadMinRep; --d)
    if (rep % d == 0) return d;
  return 1;
}

// One contiguous run of blocks of one (sequence, kv head, class): the part of it that one group works on.
struct Segment {
  int32_t b, h, cls, ntok;   // ntok: valid tokens from the first block of this piece to the end of the
                             // (sequence, kv head, class) run; may exceed nblk * 64
  int32_t blk0;              // first block, index into the class buffer
  int32_t nblk;
  int32_t gblk0;             // first block in the global order
  int32_t pid0;              // partial id of the first worker whose own range touches this segment
};

// Everything a decode workgroup needs to start streaming, in one 64-byte record.
struct WorkerRec {
  int32_t g0, g1;            // its own block range [g0, g1) of the global order
  int32_t seg0;              // index of the segment holding g0
  int32_t pid0;              // partial id of its piece of segment seg0 (in later segments it is the first visitor)
  Segment first;             // copy of segments[seg0]
  int32_t group;             // index of its GroupRec and of the group's ticket counter
  int32_t rank_nps;          // position inside the group | (GroupRec::nps << 16)
  int32_t ngran, pseg0;      // copies of the GroupRec fields, so that a worker starts from one record
};
static_assert(sizeof(WorkerRec) == 64, "WorkerRec is one 64-byte line");

// A group of consecutive workers shares a pool: the tail of the group's block range, handed out one
// loop iteration at a time through an atomic ticket counter, so that workers that finish their own
// range early take over work from slower ones.
struct GroupRec {
  int32_t ngran;             // tickets 0 .. ngran-1 are valid; 0 = the group has no pool
  int32_t pseg0;             // index of its first PoolSeg
  int32_t nps;               // number of PoolSegs (<= kMaxPoolSegments)
  int32_t nworkers;
  int32_t counter;           // index of its ticket counter (times kCounterStride)
  int32_t pad[3];
};
static_assert(sizeof(GroupRec) == 32, "GroupRec layout");

// The part of a pool that lies inside one segment.  Ticket t with gran0 <= t < gran0 + ceil(nunits / J)
// stands for units [unit0 + (t - gran0) * J, + J) of the segment, J = kIterUnits[class].
struct PoolSeg {
  int32_t seg;               // segment index
  int32_t unit0;             // first unit, counted from the start of the segment (a unit = what a wave handles at a
                             // time: 32 tokens at head_dim 128, 64 at head_dim 64)
  int32_t nunits;
  int32_t gran0;             // first ticket of this part
  int32_t slot0;             // partial id of rank 0; rank r < nslots of the group writes slot0 + r
  int32_t nslots;            // ranks that can start a partial state here: those whose own range ends in an
                             // earlier segment (the others arrive with the state of this segment)
  int32_t pad[2];
};
static_assert(sizeof(PoolSeg) == 32, "PoolSeg layout");

// One 64-token block of the packed cache as the reorder+quantize kernel sees it (one record per
// block, class by class in (b, h, block) order, i.e. in the order of the class buffers).
struct RQItem {
  int64_t ragged_row;        // row index of the block's first token in the ragged source layout
  int32_t b, h;
  int32_t t0;                // source token of row 0 if the block's rows are consecutive source tokens, else -1
  int32_t cls_nvalid;        // class | valid rows << 8
  int32_t j;                 // block index inside its (b, h, class) run
  int32_t pad;
};
static_assert(sizeof(RQItem) == 32, "RQItem layout");

struct PlanHeader {
  uint32_t magic, version;
  int32_t batch, num_q_heads, num_kv_heads, head_dim, chunk_size, group_size;
  int32_t rep;               // Hq / Hkv
  int32_t work_heads;        // heads of the decode work split: Hkv, or Hq where every query head is served by a wave
                             // of its own (vector-ALU-only plans, and Hq / Hkv beyond what the matrix kernel takes):
                             // Segment::h and the (sequence, head) ranges of partial ids count in these
  int32_t work_rep;          // query heads one workgroup serves: Hq / work_heads
  int32_t num_workers, num_segments, num_partials;
  int32_t total_gblocks;
  int32_t v_layout;          // 0: V blocks hold token rows like K; 1: token quads (2 to 8 query heads per kv head)
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
  int32_t off_class_tokens;   // int32 [B][4]
  int32_t off_class_chunk0;   // int32 [B][4]  first position in perm_b of class c
  int32_t off_blk_base;       // int32 [B+1][4] first block of sequence b in class buffer c
  int32_t off_nblk;           // int32 [B][4]  blocks per head that hold tokens
  int32_t off_run_blocks;     // int32 [B][4]  blocks per head the run is laid out with (>= the above: FP16 runs with
                              //               room for tokens that are folded in later)
  int32_t off_segments;       // Segment [num_segments]
  int32_t append_capacity;    // tokens per sequence the append buffers hold (0 = none)
  int32_t off_worker_rec;     // WorkerRec [num_workers]
  int32_t off_group_rec;      // GroupRec [num_groups]
  int32_t off_pool_seg;       // PoolSeg [num_pool_segs]
  int32_t off_counters;       // uint32 [num_groups * kCounterStride], zero; the only part kernels write
  int32_t num_groups, num_pool_segs;
  int32_t append_blocks;      // blocks per (sequence, kv head) in the append buffers
  int32_t off_bh_off;         // int32 [B*Hkv + 1] prefix: (b, kv head) owns partial ids bh_off[bh] .. bh_off[bh+1]-1;
                              // with append buffers the last append_slices ids of each range are those of the appended tokens
  int32_t off_rq_items;       // RQItem [sum of class_blocks]
  int32_t append_slices;      // workgroups (and partial ids) per (sequence, kv head) for the appended tokens
  int64_t ws_status_off;      // byte offset, inside the decode workspace, of int32 [B * Hq]: per (sequence, query
                              // head) tokens covered by the last call's partial states minus tokens of the sequence
                              // (0 = every token was attended to exactly once)
};

// Token-quad form of a V block: byte offset, inside the block, of the half-word that holds token i
// (0..63) of lane j's channels e .. e + per - 1 in the 64-channel half h, where per = 16 / bits values
// fill a half-word and ph = pieces of 16 bytes per 64-channel half of a row (bits / 2).  Channel of (h, j, e):
// 64 h + 32 (e / 8) + 8 j + e % 8.
__host__ __device__ inline uint32_t quad_halfword_offset(int ph, int per, int i, int h, int j, int e) {
  const int w = 2 * (e / per) + ((i & 3) >> 1);
  return uint32_t(((ph * h + (w >> 2)) * kTB + ((i & ~3) | j)) * 16 + (w & 3) * 4 + 2 * (i & 1));
}

template <typename T>
__host__ __device__ inline const T* plan_array(const void* blob, int32_t off) {
  return reinterpret_cast<const T*>(static_cast<const char*>(blob) + off);
}

}  // namespace cocktail

// Internal: what the two decode kernels share - the kernel arguments, buffer-resource loads, the register
// stages of the packed classes and the stream of work pieces a worker walks through.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"
#include "plan.h"

namespace cocktail {


constexpr int DH = 64;                      // channels per lane, for every head_dim
// Geometry of a wave for head_dim HD (64 or 128).  A lane always works on 64 channels of one token; a token
// is owned by HD / 64 lanes, so a wave handles 64 tokens at a time at head_dim 64 (a whole block) and 32 at
// head_dim 128 (half a block, each lane pair splitting the channels).
template <int HD>
struct Geo {
  static_assert(HD == 64 || HD == 128, "kernels are built for head_dim 64 and 128");
  static constexpr int LPT = HD / DH;         // lanes per token
  static constexpr int UT = 64 / LPT;         // tokens per unit: what one wave handles at a time
  static constexpr int UPB = kTB / UT;        // units per 64-token block
};
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleThreshold = 8.0f;   // log2 units
constexpr float kTwo24 = 16777216.0f;
constexpr int J2 = COCKTAIL_J2;    // INT2 units in flight per wave
constexpr int J4 = COCKTAIL_J4;    // INT4 units in flight per wave
constexpr int J8 = COCKTAIL_J8;    // INT8 units in flight per wave
constexpr int J16 = COCKTAIL_J16;  // FP16 units in flight per wave

struct DecodeParams {
  const WorkerRec* recs;    // [num_workers]
  const Segment* segs;      // [num_segments]
  const PoolSeg* psegs;     // [num_pool_segs]
  uint32_t* counters;       // [num_groups * kCounterStride] ticket counters, zero between calls
  const int32_t* bh_off;    // [B*Hkv + 1] (sequence, kv head) owns the partial ids bh_off[bh] .. bh_off[bh+1]-1
  const int32_t* seq_len;   // [B] context tokens per sequence
  int32_t* status;          // [B*Hq] written by the merge: 0, or how far the tokens covered by the partials are off
  const uint32_t* q;        // fp16 [B][Hq][head_dim] viewed as dwords
  const char* k[kNumClasses];
  const char* v[kNumClasses];
  const char* k_app;        // append buffers: [B*Hkv][app_blocks] FP16 blocks, or NULL
  const char* v_app;
  float* ws;                // [num_partials][rep][head_dim + 4]
  _Float16* out;            // [B][Hq][head_dim]
  float* lse;               // [B][Hq] or NULL
  float scale_log2;         // sm_scale * log2(e)
  int32_t rep, num_q_heads, num_kv_heads, num_groups;   // rep, num_kv_heads: of the work split (PlanHeader::work_rep, work_heads)
  int32_t kv_share;         // work heads that share one kv head of the cache (1, or Hq / Hkv with one wave per query head)
  int32_t num_workers;      // workgroups behind these serve the appended tokens, app_slices per (sequence, kv head)
  int32_t num_appended, app_blocks;   // tokens appended to every sequence (used if `appended` is NULL), blocks per (b, kv head)
  const int32_t* appended;  // [B] tokens appended per sequence, or NULL
  int32_t app_capacity, app_slices;   // tokens per sequence the append buffers hold; workgroups per (b, kv head) for them
#ifdef COCKTAIL_TRACE
  uint64_t* trace;          // [num_workers][4]: start, end (100 MHz ticks), hw id, xcc id
#endif
};

// The kernel keeps almost everything that describes its work in scalar registers.  To leave room
// there, the kernel arguments are not held in registers for the whole kernel: code that needs one
// of the rarely used pointers reads it from the kernel argument segment again.
typedef const __attribute__((address_space(4))) DecodeParams* kparams_t;
__device__ __forceinline__ kparams_t kparams() {
  uint64_t p = reinterpret_cast<uint64_t>(__builtin_amdgcn_kernarg_segment_ptr());
  asm volatile("" : "+s"(p));   // a fresh pointer every time: loads through it are not kept alive
  return reinterpret_cast<kparams_t>(p);
}

// A run of blocks is addressed through a buffer resource: every load is
// buffer_load(resource, lane offset in a VGPR, unit/piece offset in an SGPR), so a lane needs
// one address register per tensor kind, and reads past `bytes` return zero instead of faulting.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const char* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, bytes, 0x00020000);
}
// Cache policy of the K/V loads.  Every byte of a large cache is read exactly once per call, so the loads
// are marked non-temporal (they do not displace anything in the L2 and the memory-side cache, which on
// MI355X is worth 10 % of HBM throughput); shapes in which several workgroups walk the blocks of one kv head,
// and small caches that stay resident between calls, use the default policy.
constexpr int kAuxDefault = 0, kAuxNonTemporal = 2;
typedef __attribute__((address_space(3))) char* lds_ptr_t;   // a wave-uniform address in shared memory
constexpr int64_t kNonTemporalMinBytes = int64_t(64) << 20;   // packed K+V bytes of one call
template <int AUX>
__device__ __forceinline__ u32x4 load16(rsrc_t rs, uint32_t voff, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, AUX);
}

__device__ __forceinline__ float dot2(uint32_t qpair, uint32_t kv, float acc) {
  return __builtin_amdgcn_fdot2(as_h2(qpair), as_h2(kv), acc, false);
}

// acc + f32 * (low | high half of hv as fp16): compiles to v_fma_mix_f32
__device__ __forceinline__ float fma_lo(float a, uint32_t hv, float acc) {
  return acc + a * static_cast<float>(as_h2(hv).x);
}
__device__ __forceinline__ float fma_hi(float a, uint32_t hv, float acc) {
  return acc + a * static_cast<float>(as_h2(hv).y);
}

__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// Marks a value as wave-uniform (it is: everything derived from the plan is), so that it lives in
// scalar registers and buffer loads need no per-lane resource handling.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ const char* uni(const char* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v)), hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
  return reinterpret_cast<const char*>((uint64_t(hi) << 32) | lo);
}
__device__ __forceinline__ Segment uni(const Segment& x) {
  Segment y;
  y.b = uni(x.b), y.h = uni(x.h), y.cls = uni(x.cls), y.ntok = uni(x.ntok);
  y.blk0 = uni(x.blk0), y.nblk = uni(x.nblk), y.gblk0 = uni(x.gblk0), y.pid0 = uni(x.pid0);
  return y;
}

// Zero-instruction anchor: the value must exist in a VGPR at this point of the program order.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }

template <int NGH>
struct LaneState {
  float acc[DH];       // sum_t p_t * (scale * code | value) for this lane's 64 channels
  float zacc[NGH];     // sum_t p_t * zero_tg for this lane's groups
  float m, l;
};

// ---------------------------------------------------------------- quantised classes
// A word holds 32/BITS codes; even channels in the low half-word, odd ones in the high
// half-word.  Masking field k of both half-words of `w` or `w >> 8` leaves two fp16
// subnormals  code * 2^(BITS*k - 24)  for the channel pair (2f, 2f+1), f = 4*half + k
// (INT2), 2*half + k (INT4) or half (INT8, one field per byte).
template <int HD, int BITS, int G>
struct QuantClass {
  static constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  static constexpr int PH = DH * BITS / 128;        // 16-byte pieces per lane and unit
  static constexpr int NG = HD / G;
  static constexpr int NGH = G < DH ? DH / G : 1;   // groups a lane touches
  static constexpr int GL = G < DH ? G : DH;        // channels of a lane that share one group
  static constexpr int CPW = 32 / BITS;             // channels per word
  static constexpr int NPOS = 8 / BITS;             // fields per byte: 4 (INT2), 2 (INT4) or 1 (INT8)
  static constexpr int ROWB = HD * BITS / 8;
  static constexpr int BLOCKB = kTB * (ROWB + 4 * NG);
  static constexpr int J = BITS == 2 ? J2 : BITS == 4 ? J4 : J8;
  static constexpr uint32_t MASK0 = (BITS == 2) ? 0x00030003u : (BITS == 4) ? 0x000F000Fu : 0x00FF00FFu;

  struct Stage {              // one lane's share of one unit of K or V
    u32x4 pc[PH];
    uint32_t meta[NGH];
  };

  // per-lane byte offsets of the code pieces and of the scale/zero pairs inside a unit
  __device__ static __forceinline__ uint32_t code_voff(int t, int h) { return (PH * h * kTB + t) * 16u; }
  __device__ static __forceinline__ uint32_t meta_voff(int t, int h) {
    return (t * NG + (h * DH) / G) * 4u;   // the lane's first group
  }

  // unit u of the run = tokens [UT u, UT u + UT): block u / UPB, and which part of its token slots
  template <int AUX>
  __device__ static __forceinline__ void load(Stage& s, rsrc_t rs, int u, uint32_t vc, uint32_t vm) {
    const uint32_t boff = uint32_t(u / UPB) * BLOCKB;
    const uint32_t sub = uint32_t(u % UPB);
#pragma unroll
    for (int p = 0; p < PH; ++p) s.pc[p] = load16<AUX>(rs, vc, boff + sub * (UT * 16) + p * (kTB * 16));
    const uint32_t moff = boff + kTB * ROWB + sub * (UT * 4 * NG);
    if constexpr (NGH == 2) {
      const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, vm, moff, AUX);
      s.meta[0] = t.x, s.meta[1] = t.y;
    } else {
      s.meta[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, vm, moff, AUX);
    }
  }

  // The same unit fetched into shared memory instead (workgroups whose waves share their K/V units): the
  // image is what the lanes of one wave would hold in registers, piece p of lane l at p*1024 + l*16 and
  // scale/zero dword g of lane l at PH*1024 + g*256 + l*4; the loads write it without passing through registers.
  static constexpr int LDS_UNIT = PH * 1024 + NGH * 256;
  template <int AUX>
  __device__ static __forceinline__ void load_lds(lds_ptr_t dst, rsrc_t rs, int u, uint32_t vc, uint32_t vm) {
    const uint32_t boff = uint32_t(u / UPB) * BLOCKB;
    const uint32_t sub = uint32_t(u % UPB);
#pragma unroll
    for (int p = 0; p < PH; ++p)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst + p * 1024, 16, vc, boff + sub * (UT * 16) + p * (kTB * 16), 0, AUX);
    const uint32_t moff = boff + kTB * ROWB + sub * (UT * 4 * NG);
#pragma unroll
    for (int g = 0; g < NGH; ++g) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst + PH * 1024 + g * 256, 4, vm + g * 4, moff, 0, AUX);
  }
  __device__ static __forceinline__ void read_lds(Stage& s, const char* src, int lane) {
#pragma unroll
    for (int p = 0; p < PH; ++p) s.pc[p] = *reinterpret_cast<const u32x4*>(src + p * 1024 + lane * 16);
#pragma unroll
    for (int g = 0; g < NGH; ++g) s.meta[g] = *reinterpret_cast<const uint32_t*>(src + PH * 1024 + g * 256 + lane * 4);
  }

  // this lane's half of q.k^ (natural units, before the softmax scale)
  __device__ static __forceinline__ float half_logit(const Stage& s, const uint32_t (&q)[DH / 2],
                                                     const float (&qsum)[NGH]) {
    float ga[NGH][NPOS];
#pragma unroll
    for (int g = 0; g < NGH; ++g)
#pragma unroll
      for (int k = 0; k < NPOS; ++k) ga[g][k] = 0.f;
#pragma unroll
    for (int p = 0; p < PH; ++p)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int cb = (p * 4 + wi) * CPW;          // first local channel of the word
        const uint32_t w0 = s.pc[p][wi];
        const uint32_t w1 = w0 >> 8;
#pragma unroll
        for (int k = 0; k < NPOS; ++k) {
          const uint32_t mask = MASK0 << (BITS * k);
          ga[cb / GL][k] = dot2(q[cb / 2 + k], w0 & mask, ga[cb / GL][k]);
          ga[cb / GL][k] = dot2(q[cb / 2 + NPOS + k], w1 & mask, ga[cb / GL][k]);
        }
      }
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < NGH; ++g) {
      float t = ga[g][NPOS - 1];
#pragma unroll
      for (int k = NPOS - 2; k >= 0; --k) t = t * (1.0f / float(1 << BITS)) + ga[g][k];
      // t = sum_d q_d code_d * 2^-24 over the lane's channels of group g
      const h2 mz = as_h2(s.meta[g]);
      sum += (static_cast<float>(mz.x) * kTwo24) * t + static_cast<float>(mz.y) * qsum[g];
    }
    return sum;
  }

  __device__ static __forceinline__ void accumulate(const Stage& s, float p, LaneState<NGH>& st) {
    float ps[NGH][NPOS];
#pragma unroll
    for (int g = 0; g < NGH; ++g) {
      const h2 mz = as_h2(s.meta[g]);
      float f = p * static_cast<float>(mz.x) * kTwo24;
#pragma unroll
      for (int k = 0; k < NPOS; ++k) {
        ps[g][k] = f;
        f *= 1.0f / float(1 << BITS);
      }
      st.zacc[g] += p * static_cast<float>(mz.y);
    }
#pragma unroll
    for (int p_ = 0; p_ < PH; ++p_)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int cb = (p_ * 4 + wi) * CPW;
        const uint32_t w0 = s.pc[p_][wi];
        const uint32_t w1 = w0 >> 8;
#pragma unroll
        for (int k = 0; k < NPOS; ++k) {
          const uint32_t mask = MASK0 << (BITS * k);
          const uint32_t x0 = w0 & mask, x1 = w1 & mask;
          const float f = ps[cb / GL][k];
          st.acc[cb + 2 * k] = fma_lo(f, x0, st.acc[cb + 2 * k]);
          st.acc[cb + 2 * k + 1] = fma_hi(f, x0, st.acc[cb + 2 * k + 1]);
          st.acc[cb + 2 * (NPOS + k)] = fma_lo(f, x1, st.acc[cb + 2 * (NPOS + k)]);
          st.acc[cb + 2 * (NPOS + k) + 1] = fma_hi(f, x1, st.acc[cb + 2 * (NPOS + k) + 1]);
        }
        // Pin the word's accumulators here: without it the optimiser sinks all multiply-adds of a
        // stage below the unpacking of every word and the masked temporaries pile up.
#pragma unroll
        for (int i = 0; i < CPW; ++i) pin(st.acc[cb + i]);
      }
  }
};

// ---------------------------------------------------------------------- FP16 class
template <int HD, int G>
struct HalfClass {
  static constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  static constexpr int PH = 8;
  static constexpr int NG = HD / G;
  static constexpr int NGH = G < DH ? DH / G : 1;
  static constexpr int BLOCKB = kTB * 2 * HD;
  static constexpr int J = J16;

  struct Stage {
    u32x4 pc[PH];
  };
  __device__ static __forceinline__ uint32_t code_voff(int t, int h) { return (PH * h * kTB + t) * 16u; }
  __device__ static __forceinline__ uint32_t meta_voff(int, int) { return 0; }

  template <int AUX>
  __device__ static __forceinline__ void load(Stage& s, rsrc_t rs, int u, uint32_t vc, uint32_t) {
    const uint32_t boff = uint32_t(u / UPB) * BLOCKB + uint32_t(u % UPB) * (UT * 16);
#pragma unroll
    for (int p = 0; p < PH; ++p) s.pc[p] = load16<AUX>(rs, vc, boff + p * (kTB * 16));
  }

  static constexpr int LDS_UNIT = PH * 1024;   // see QuantClass::load_lds
  template <int AUX>
  __device__ static __forceinline__ void load_lds(lds_ptr_t dst, rsrc_t rs, int u, uint32_t vc, uint32_t) {
    const uint32_t boff = uint32_t(u / UPB) * BLOCKB + uint32_t(u % UPB) * (UT * 16);
#pragma unroll
    for (int p = 0; p < PH; ++p) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst + p * 1024, 16, vc, boff + p * (kTB * 16), 0, AUX);
  }
  __device__ static __forceinline__ void read_lds(Stage& s, const char* src, int lane) {
#pragma unroll
    for (int p = 0; p < PH; ++p) s.pc[p] = *reinterpret_cast<const u32x4*>(src + p * 1024 + lane * 16);
  }

  __device__ static __forceinline__ float half_logit(const Stage& s, const uint32_t (&q)[DH / 2],
                                                     const float (&)[NGH]) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int p = 0; p < PH; ++p) {
      a0 = dot2(q[p * 4 + 0], s.pc[p][0], a0);
      a1 = dot2(q[p * 4 + 1], s.pc[p][1], a1);
      a0 = dot2(q[p * 4 + 2], s.pc[p][2], a0);
      a1 = dot2(q[p * 4 + 3], s.pc[p][3], a1);
    }
    return a0 + a1;
  }

  __device__ static __forceinline__ void accumulate(const Stage& s, float p, LaneState<NGH>& st) {
#pragma unroll
    for (int pi = 0; pi < PH; ++pi) {
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int d = (pi * 4 + wi) * 2;
        st.acc[d] = fma_lo(p, s.pc[pi][wi], st.acc[d]);
        st.acc[d + 1] = fma_hi(p, s.pc[pi][wi], st.acc[d + 1]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) pin(st.acc[pi * 8 + i]);
    }
  }
};

// ------------------------------------------------------------------ the worker's stream
// One loop iteration's worth of work: up to J consecutive units of one segment.  Wave-uniform.
struct Piece {
  int nu;          // units; 0 = the stream has ended
  int us;          // first unit, counted from the start of the segment
  int valid;       // valid tokens among the nu * 32
  int cls;
  int fresh;       // 1 = the worker's first piece in this segment: a new partial state starts here
  int pid;         // partial id of that state (meaningful when fresh)
};                 // the segment it lies in is the stream's current one (blk0, nblk, qrow there)

__device__ __forceinline__ int iter_units(int cls) { return cls == 0 ? J2 : cls == 1 ? J4 : cls == 2 ? J8 : J16; }

// A ticket from the group's counter.  The value is only needed a few loop iterations later; it
// travels through the vector memory pipeline like any load and is picked up with readfirstlane.
// The add is a buffer atomic over a 4-byte resource with one offset per lane, so only lane 0 is in
// range and performs it (out-of-range lanes are dropped by the bounds check): no divergent branch.
__device__ __forceinline__ uint32_t request_ticket(int counter, int lane) {
  uint32_t* c = kparams()->counters + counter * kCounterStride;
  const rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(c, 0, 4, 0x00020000);
  return uint32_t(__builtin_amdgcn_raw_ptr_buffer_atomic_add_i32(1, rs, lane * 4, 0, /*sc1: device scope*/ 16));
}

// Yields the pieces of one worker: first its own block range front to back, then pieces of the
// group's pool, one ticket each, until the tickets run out.  Segments are visited in ascending
// order, so every segment is entered at most once.
template <int HD>
struct Stream {
  static constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  int u, u1;          // own range: cursor and end in global units (UPB per block)
  int s;              // index of the current segment; the fields below describe it
  int cls, ntok, blk0, nblk, gu0, qrow;   // gu0: first global unit of the segment
  int pid;            // partial id of this worker's own piece of the current segment
  int last_seg;       // segment of the previous piece
  int ngran, nps, pseg0, rank, counter;
  int pi;             // current pool part (index relative to pseg0), -1 before the first
  int p_unit0, p_nunits, p_gran0, p_gran1, p_slot0;
  uint32_t tk0, tk1;  // tickets in flight (lane 0 holds the value)
  uint32_t used;      // pool parts for which this worker started a partial state
  int phase;          // 0 own range, tickets not requested; 1 own range, requested; 2 pool; 3 done

  __device__ __forceinline__ void enter(const Segment& g, int index) {
    kparams_t kp = kparams();
    s = index;
    cls = uni(g.cls), ntok = uni(g.ntok), blk0 = uni(g.blk0), nblk = uni(g.nblk), gu0 = UPB * uni(g.gblk0);
    pid = uni(g.pid0);   // whoever enters a segment from its start is its first visitor
    qrow = uni(g.b) * kp->num_q_heads + uni(g.h) * kp->rep;
  }

  __device__ __forceinline__ void init(const WorkerRec& rec) {
    u = UPB * uni(rec.g0), u1 = UPB * uni(rec.g1);
    enter(rec.first, uni(rec.seg0));
    pid = uni(rec.pid0);   // the first segment is usually entered somewhere in the middle
    if (u >= u1) s = -1;   // no own range: `first` describes nothing, the first pool piece enters its segment
    last_seg = -1;
    const int rn = uni(rec.rank_nps);
    ngran = uni(rec.ngran), nps = rn >> 16, pseg0 = uni(rec.pseg0), rank = rn & 0xffff;
    counter = uni(rec.group);
    pi = -1, p_unit0 = p_nunits = p_gran0 = p_gran1 = p_slot0 = 0;
    tk0 = tk1 = 0, used = 0;
    phase = 0;
  }

  // A stream over one run of blocks of class `c` only (the appended tokens): no pool, one partial state.
  __device__ __forceinline__ void init_run(int c, int tokens, int first_block, int blocks, int query_row, int partial) {
    u = 0, u1 = (tokens + UT - 1) / UT;
    s = 0;
    cls = c, ntok = tokens, blk0 = first_block, nblk = blocks, gu0 = 0;
    qrow = query_row;
    pid = partial;
    last_seg = -1;
    ngran = 0, nps = 0, pseg0 = 0, rank = 0, counter = 0;
    pi = -1, p_unit0 = p_nunits = p_gran0 = p_gran1 = p_slot0 = 0;
    tk0 = tk1 = 0, used = 0;
    phase = 0;
  }

  __device__ __forceinline__ void fill(Piece& d, int us, int nu) {
    d.nu = nu, d.us = us;
    d.valid = max(0, min(ntok - us * UT, nu * UT));
    d.cls = cls;
    d.fresh = s != last_seg;
    last_seg = s;
  }

  __device__ __forceinline__ Piece next(int lane) {
    Piece d;
    d.nu = 0, d.us = 0, d.valid = 0, d.cls = -1, d.fresh = 0, d.pid = 0;
    if (phase <= 1) {
      // ask for the first tickets a few iterations before the own range runs out
      if (phase == 0 && ngran > 0 && u1 - u <= 3 * iter_units(cls)) {
        tk0 = request_ticket(counter, lane);
        tk1 = request_ticket(counter, lane);
        phase = 1;
      }
      if (u < u1) {
        if (u >= gu0 + UPB * nblk) enter(load_record(kparams()->segs + s + 1), s + 1);
        const int us = u - gu0;
        const int nu = min(iter_units(cls), min(u1 - gu0, UPB * nblk) - us);
        if (nu <= 0) {   // cannot happen with a plan written by cocktail_plan; guarantees termination
          phase = 3;
          return d;
        }
        fill(d, us, nu);
        if (d.fresh) d.pid = pid;
        u += nu;
        return d;
      }
      phase = ngran > 0 ? 2 : 3;
    }
    if (phase == 2) {
      const uint32_t t = __builtin_amdgcn_readfirstlane(tk0);
      tk0 = tk1;
      tk1 = request_ticket(counter, lane);
      if (t >= uint32_t(ngran)) {
        phase = 3;
        return d;
      }
      while (pi < 0 || int(t) >= p_gran1) {
        if (++pi >= nps) {   // cannot happen with a plan written by cocktail_plan; guarantees termination
          phase = 3;
          return d;
        }
        kparams_t kp = kparams();
        const PoolSeg ps = load_record(kp->psegs + pseg0 + pi);
        const int seg = uni(ps.seg);
        p_unit0 = uni(ps.unit0), p_nunits = uni(ps.nunits), p_gran0 = uni(ps.gran0), p_slot0 = uni(ps.slot0);
        if (seg != s) enter(load_record(kp->segs + seg), seg);
        const int j = iter_units(cls);
        p_gran1 = p_gran0 + (p_nunits + j - 1) / j;
      }
      const int j = iter_units(cls);
      const int us = p_unit0 + (int(t) - p_gran0) * j;
      const int nu = min(j, p_unit0 + p_nunits - us);
      if (nu <= 0) {
        phase = 3;
        return d;
      }
      fill(d, us, nu);
      if (d.fresh) {
        d.pid = p_slot0 + rank;
        used |= 1u << pi;
      }
    }
    return d;
  }
};

// Tokens appended to sequence b so far (never more than the append buffers hold).
__device__ __forceinline__ int appended_count(int b) {
  kparams_t kp = kparams();
  const int n = kp->appended ? kp->appended[b] : kp->num_appended;
  return min(max(n, 0), kp->app_capacity);
}

// The part of an append run that workgroup `idx` behind the regular workers attends to.
struct AppendSlice {
  int bh, tokens, first_block, blocks, qrow, pid;
};
__device__ __forceinline__ AppendSlice append_slice(int idx) {
  kparams_t kp = kparams();
  AppendSlice a;
  const int slices = kp->app_slices, sl = idx % slices;
  a.bh = idx / slices;
  const int b = a.bh / kp->num_kv_heads;
  const int first = sl * kAppendSliceBlocks;
  a.tokens = uni(min(max(appended_count(b) - first * kTB, 0), kAppendSliceBlocks * kTB));
  a.blocks = min(kAppendSliceBlocks, kp->app_blocks - first);
  // the append buffers are laid out by (sequence, kv head of the cache)
  a.first_block = (b * (kp->num_kv_heads / kp->kv_share) + (a.bh % kp->num_kv_heads) / kp->kv_share) * kp->app_blocks + first;
  a.qrow = b * kp->num_q_heads + (a.bh % kp->num_kv_heads) * kp->rep;
  a.pid = uni(kp->bh_off[a.bh + 1]) - slices + sl;
  return a;
}

// The neutral partial state (weight zero in the merge) for a slot nobody had tokens for.
template <int HD>
__device__ __forceinline__ void write_neutral(int slot, int r, int lane) {
  kparams_t kp = kparams();
  float* out = kp->ws + (int64_t(slot) * kp->rep + r) * (HD + kPartialFloats);
  if (lane == 0) out[0] = kNegBig, out[1] = 0.f, out[2] = 0.f;   // covers no tokens
#pragma unroll
  for (int i = 0; i < HD / 64; ++i) out[kPartialFloats + 64 * i + lane] = 0.f;
}

// Launch the partial-state kernels for head_dim HD (one translation unit per head_dim and kernel family):
// one query head per wave on the vector ALU; 2 to 8 query heads per kv head on matrix instructions, `grid`
// workgroups of one wave (up to 4 heads) or two waves (5 to 8).  int8: the cache has an INT8 class.
template <int HD>
hipError_t launch_decode_heads(const DecodeParams& p, int group_size, bool non_temporal, bool int8, int grid, hipStream_t st);
template <int HD>
hipError_t launch_decode_quads(const DecodeParams& p, int group_size, bool non_temporal, bool int8, int grid, hipStream_t st);

}  // namespace cocktail

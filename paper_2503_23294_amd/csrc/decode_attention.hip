// Decode side of Alg. 1 (Sec. III-C): single-query attention over the INT2, INT4
// and FP16 classes of the packed cache.
//
// Design (gfx950, wave64):
//  * The host planner puts all 64-token blocks of a layer into one global order and cuts it into
//    groups of a few workers.  A worker (workgroup) streams its own block range and then takes
//    pieces of the group's shared pool through an atomic ticket counter, so that the workers of a
//    group finish together; it emits one partial softmax state per (sequence, kv head) segment it
//    touches.
//  * Inside a wave a token is owned by a PAIR of lanes: lane l works on token
//    l % 32 of a 32-token unit and on channels [64*(l/32), 64*(l/32)+64).  The block
//    layout stores the j-th 16-byte piece of all 64 tokens contiguously, so each
//    half-wave reads one contiguous 512-byte run per load instruction, and the q.k
//    dot product needs a single cross-lane add per token.  A lane keeps 64 output
//    accumulators and its half of the query in registers; the kernel stays below
//    256 VGPRs so that two waves share every SIMD and one wave's loads hide behind
//    the other's arithmetic.
//  * Codes are expanded without any conversion: a code field masked out of a
//    half-word IS an fp16 subnormal of value code * 2^(pos-24), which v_dot2_f32_f16
//    and v_fma_mix_f32 consume exactly; the power of two is folded into per-group
//    factors.  Dequantisation is folded too:
//      q.k^      = sum_g scale_g * (q.code)_g + zero_g * sum(q_g)
//      sum p v^  = sum_t (p_t scale_tg) code_t + sum_t p_t zero_tg
//  * Loads go through buffer resources (one VGPR of address per lane) and are
//    software pipelined by hand: J register stages of K units and J of V units are
//    refilled one loop iteration ahead of the arithmetic, with the units of whatever
//    piece comes next (same segment, next segment, or a pool piece).
//  * Softmax is online per lane pair: logits of J units, one lazy rescale when the
//    reference maximum grows by more than 2^8, then the V pass.  (m, l, o[D])
//    partials go to the workspace and a second small kernel merges them exactly
//    (the softmax-weighted sum does not depend on how tokens are grouped, Eq. 4-5).
//  * Grouped-query attention: the Hq/Hkv query heads of a kv head run as separate
//    waves of one workgroup on the same blocks, so the second to last read hits cache.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>

#include "common.h"
#include "plan.h"

namespace cocktail {

constexpr int D = 128;
constexpr int DH = D / 2;                   // channels per lane
constexpr int UT = 32;                      // tokens per unit (half a block)
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleThreshold = 8.0f;   // log2 units
constexpr float kTwo24 = 16777216.0f;
#ifndef COCKTAIL_J2
#define COCKTAIL_J2 4
#endif
#ifndef COCKTAIL_J4
#define COCKTAIL_J4 2
#endif
#ifndef COCKTAIL_J16
#define COCKTAIL_J16 1
#endif
constexpr int J2 = COCKTAIL_J2;    // INT2 units in flight per wave
constexpr int J4 = COCKTAIL_J4;    // INT4 units in flight per wave
constexpr int J16 = COCKTAIL_J16;  // FP16 units in flight per wave

struct DecodeParams {
  const WorkerRec* recs;    // [num_workers]
  const Segment* segs;      // [num_segments]
  const PoolSeg* psegs;     // [num_pool_segs]
  uint32_t* counters;       // [num_groups * kCounterStride] ticket counters, zero between calls
  const int32_t* bh_off;    // [B*Hkv + 1] (sequence, kv head) owns the partial ids bh_off[bh] .. bh_off[bh+1]-1
  const uint32_t* q;        // fp16 [B][Hq][D] viewed as dwords
  const char* k[3];
  const char* v[3];
  const char* k_app;        // append buffers: [B*Hkv][app_blocks] FP16 blocks, or NULL
  const char* v_app;
  float* ws;                // [num_partials][rep][D + 2]
  _Float16* out;            // [B][Hq][D]
  float* lse;               // [B][Hq] or NULL
  float scale_log2;         // sm_scale * log2(e)
  int32_t rep, num_q_heads, num_kv_heads, num_groups;
  int32_t num_workers;      // workgroups behind these serve the appended tokens, one per (sequence, kv head)
  int32_t num_appended, app_blocks;
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
// MI355X is worth 10 % of HBM throughput); grouped-query shapes, whose waves re-read each other's lines
// from the L2, and small caches that stay resident between calls use the default policy.
constexpr int kAuxDefault = 0, kAuxNonTemporal = 2;
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
// (INT2) or 2*half + k (INT4).
template <int BITS, int G>
struct QuantClass {
  static constexpr int PH = D * BITS / 256;         // 16-byte pieces per lane and unit
  static constexpr int NG = D / G;
  static constexpr int NGH = NG >= 2 ? NG / 2 : 1;  // groups a lane touches
  static constexpr int GL = G < DH ? G : DH;        // channels of a lane that share one group
  static constexpr int CPW = 32 / BITS;             // channels per word
  static constexpr int NPOS = 8 / BITS;             // fields per byte: 4 (INT2) or 2 (INT4)
  static constexpr int ROWB = D * BITS / 8;
  static constexpr int BLOCKB = kTB * (ROWB + 4 * NG);
  static constexpr int J = BITS == 2 ? J2 : J4;
  static constexpr uint32_t MASK0 = (BITS == 2) ? 0x00030003u : 0x000F000Fu;

  struct Stage {              // one lane's share of one unit of K or V
    u32x4 pc[PH];
    uint32_t meta[NGH];
  };

  // per-lane byte offsets of the code pieces and of the scale/zero pairs inside a unit
  __device__ static __forceinline__ uint32_t code_voff(int t, int h) { return (PH * h * kTB + t) * 16u; }
  __device__ static __forceinline__ uint32_t meta_voff(int t, int h) {
    return NG >= 2 ? (t * NG + h * NGH) * 4u : t * 4u;
  }

  // unit u of the run = tokens [32u, 32u+32): block u/2, first or second half of its token slots
  template <int AUX>
  __device__ static __forceinline__ void load(Stage& s, rsrc_t rs, int u, uint32_t vc, uint32_t vm) {
    const uint32_t boff = uint32_t(u >> 1) * BLOCKB;
    const uint32_t sub = uint32_t(u & 1);
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
template <int G>
struct HalfClass {
  static constexpr int PH = 8;
  static constexpr int NG = D / G;
  static constexpr int NGH = NG >= 2 ? NG / 2 : 1;
  static constexpr int BLOCKB = kTB * 2 * D;
  static constexpr int J = J16;

  struct Stage {
    u32x4 pc[PH];
  };
  __device__ static __forceinline__ uint32_t code_voff(int t, int h) { return (PH * h * kTB + t) * 16u; }
  __device__ static __forceinline__ uint32_t meta_voff(int, int) { return 0; }

  template <int AUX>
  __device__ static __forceinline__ void load(Stage& s, rsrc_t rs, int u, uint32_t vc, uint32_t) {
    const uint32_t boff = uint32_t(u >> 1) * BLOCKB + uint32_t(u & 1) * (UT * 16);
#pragma unroll
    for (int p = 0; p < PH; ++p) s.pc[p] = load16<AUX>(rs, vc, boff + p * (kTB * 16));
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

// One lazy-rescale step of a lane's online softmax followed by p_j = 2^(s_j - m).
template <int NGH, int J>
__device__ __forceinline__ void softmax_step(const float (&s)[J], float (&p)[J], LaneState<NGH>& st) {
  float smax = s[0];
#pragma unroll
  for (int jj = 1; jj < J; ++jj) smax = fmaxf(smax, s[jj]);
  // the reference maximum only moves when it is exceeded by more than 2^8, and then for the whole
  // wave at once (to the largest logit any lane has seen): the lanes share one reference, so the
  // number of rescales per state is that of one running maximum, not of 64 independent ones
  const bool grow = smax > st.m + kRescaleThreshold;
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
    float mnew = fmaxf(smax, st.m);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mnew = fmaxf(mnew, __shfl_xor(mnew, o));
    const float alpha = __builtin_amdgcn_exp2f(st.m - mnew);
    st.m = mnew;
    st.l *= alpha;
#pragma unroll
    for (int d = 0; d < DH; ++d) st.acc[d] *= alpha;
#pragma unroll
    for (int g = 0; g < NGH; ++g) st.zacc[g] *= alpha;
  }
#pragma unroll
  for (int jj = 0; jj < J; ++jj) {
    p[jj] = __builtin_amdgcn_exp2f(s[jj] - st.m);
    st.l += p[jj];
  }
}

// Writes this wave's partial state `pid`: (m, l, o[D]) reduced over its lanes.
template <int NGH, int GL>
__device__ __forceinline__ void flush_partial(const LaneState<NGH>& st, float* red, int pid, int r, int lane) {
  kparams_t prm = kparams();
  const int rep = prm->rep;
  float mw = st.m;
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  const float f = __builtin_amdgcn_exp2f(st.m - mw);
  float lw = st.l * f;
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
  float* out = prm->ws + (int64_t(pid) * rep + r) * (D + kPartialFloats);
  if (lane == 0) {
    out[0] = mw;
    out[1] = lw;
  }
  float(*tile)[17] = reinterpret_cast<float(*)[17]>(red + r * 64 * 17);
#pragma unroll
  for (int ch = 0; ch < DH / 16; ++ch) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const int d = ch * 16 + c;
      tile[lane][c] = (st.acc[d] + st.zacc[d / GL]) * f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane (c, quarter) adds 16 rows; quarters 0,1 hold channel half 0 and quarters 2,3 half 1
    const int c = lane & 15, quarter = lane >> 4;
    float sum = 0.f;
#pragma unroll
    for (int row = 0; row < 16; ++row) sum += tile[quarter * 16 + row][c];
    sum += __shfl_xor(sum, 16);
    if ((quarter & 1) == 0) out[kPartialFloats + (quarter >> 1) * DH + ch * 16 + c] = sum;
  }
}

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

__device__ __forceinline__ int iter_units(int cls) { return cls == 0 ? J2 : cls == 1 ? J4 : J16; }

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
struct Stream {
  int u, u1;          // own range: cursor and end in global units (two per block)
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
    cls = uni(g.cls), ntok = uni(g.ntok), blk0 = uni(g.blk0), nblk = uni(g.nblk), gu0 = 2 * uni(g.gblk0);
    pid = uni(g.pid0);   // whoever enters a segment from its start is its first visitor
    qrow = uni(g.b) * kp->num_q_heads + uni(g.h) * kp->rep;
  }

  __device__ __forceinline__ void init(const WorkerRec& rec) {
    u = 2 * uni(rec.g0), u1 = 2 * uni(rec.g1);
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
        if (u >= gu0 + 2 * nblk) enter(load_record(kparams()->segs + s + 1), s + 1);
        const int us = u - gu0;
        const int nu = min(iter_units(cls), min(u1 - gu0, 2 * nblk) - us);
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

// Zeroes the partial state and loads this lane's half of the query row `qrow`.
template <int NGH, int GL>
__device__ __forceinline__ void begin_state(int qrow, int h, LaneState<NGH>& st, uint32_t (&q)[DH / 2],
                                            float (&qsum)[NGH]) {
#pragma unroll
  for (int i = 0; i < DH; ++i) st.acc[i] = 0.f;
#pragma unroll
  for (int gq = 0; gq < NGH; ++gq) st.zacc[gq] = 0.f;
  st.m = kNegBig;
  st.l = 0.f;
  const u32x4* qp = reinterpret_cast<const u32x4*>(kparams()->q + int64_t(qrow) * (D / 2) + h * (DH / 2));
#pragma unroll
  for (int i = 0; i < DH / 8; ++i) {
    const u32x4 v = qp[i];
    q[4 * i] = v.x, q[4 * i + 1] = v.y, q[4 * i + 2] = v.z, q[4 * i + 3] = v.w;
  }
#pragma unroll
  for (int gq = 0; gq < NGH; ++gq) {
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < GL / 2; ++i) a = dot2(q[gq * (GL / 2) + i], 0x3C003C00u, a);   // (1.0, 1.0)
    qsum[gq] = a;
  }
}

// Consumes the stream while its pieces belong to class CID, starting with `cur` (whose loads have
// not been issued yet); returns with `cur` = the first piece of another class, or the end piece.
//
// J register stages hold the K units and J the V units of the piece being worked on; each stage is
// refilled with the corresponding unit of the NEXT piece as soon as it has been consumed, so the
// loads of a piece are in flight during the arithmetic of the piece before it, across segment and
// pool boundaries alike.  A piece with fewer than J units leaves stages unused, and after the last
// piece of the class nothing is left to fetch: those refills address the first unit past the segment,
// which the buffer resource answers with zeros without touching memory, so the loop body has no
// branches around the loads (the zeros are masked like padding).  The accumulators live and die inside this function, one
// instance per class.
template <class CLS, int CID, int G, int AUX>
__device__ __forceinline__ void run_class(Stream& sm, Piece& cur, float* red, int r, int lane, bool app = false) {
  constexpr int NG = D / G;
  constexpr int NGH = NG >= 2 ? NG / 2 : 1;
  constexpr int GL = G < DH ? G : DH;
  constexpr int J = CLS::J;
  static_assert(J == kIterUnits[CID], "the planner cuts pool pieces to the kernel's iteration size");
  const int t = lane & 31, h = lane >> 5;
  const uint32_t vc = CLS::code_voff(t, h), vm = CLS::meta_voff(t, h);
  const char* const kbase = uni(app ? kparams()->k_app : kparams()->k[CID]);   // app: the append buffers
  const char* const vbase = uni(app ? kparams()->v_app : kparams()->v[CID]);
  const float scale_log2 = kparams()->scale_log2;
  LaneState<NGH> st;
  uint32_t q[DH / 2];
  float qsum[NGH];
  typename CLS::Stage ks[J], vs[J];
  int pid = cur.pid;
  // `cur` is the piece the stream produced last, so the stream's segment fields describe it
  rsrc_t krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  rsrc_t vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  int ru = cur.us, rn = cur.nu;   // the piece the stages are (re)filled with
  int roob = 2 * sm.nblk;         // first unit past its segment: a load from there is out of range and costs nothing
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
  sched_fence();
  begin_state<NGH, GL>(sm.qrow + r, h, st, q, qsum);   // the query arrives while the first units are on their way
  int valid = cur.valid;
  Piece nxt = sm.next(lane);
#pragma unroll 1
  while (true) {
    const bool more = nxt.nu > 0 && nxt.cls == CID;
    if (more) {
      krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      ru = nxt.us, rn = nxt.nu, roob = 2 * sm.nblk;
    } else {
      rn = 0;   // nothing follows in this class: every refill goes out of range
    }
    float s[J], p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      s[jj] = CLS::half_logit(ks[jj], q, qsum);
      sched_fence();
      CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      const float full = (s[jj] + __shfl_xor(s[jj], 32)) * scale_log2;   // both halves of the token
      s[jj] = (jj * UT + t < valid) ? full : -INFINITY;
    }
    softmax_step<NGH, J>(s, p, st);
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      CLS::accumulate(vs[jj], p[jj], st);
      sched_fence();
      CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
    if (!more || nxt.fresh) flush_partial<NGH, GL>(st, red, pid, r, lane);
    if (!more) break;
    if (nxt.fresh) {
      pid = nxt.pid;
      begin_state<NGH, GL>(sm.qrow + r, h, st, q, qsum);
    }
    valid = nxt.valid;
    nxt = sm.next(lane);
  }
  cur = nxt;
}

// The neutral partial state (weight zero in the merge) for a slot nobody had tokens for.
__device__ __forceinline__ void write_neutral(int slot, int r, int lane) {
  kparams_t kp = kparams();
  float* out = kp->ws + (int64_t(slot) * kp->rep + r) * (D + kPartialFloats);
  if (lane == 0) out[0] = kNegBig, out[1] = 0.f;
  out[kPartialFloats + lane] = 0.f;
  out[kPartialFloats + 64 + lane] = 0.f;
}

// Workgroups behind the regular workers: workgroup num_workers + bh attends to the tokens appended to
// (sequence, kv head) bh during decoding (Sec. III-A), an FP16 run of num_appended tokens in the
// append buffers, and writes the last partial of bh's range.
template <int G, int AUX>
__device__ __forceinline__ void appended_tokens(int bh, float* red, int r, int lane) {
  kparams_t kp = kparams();
  const int n = kp->num_appended;
  const int pid = uni(kp->bh_off[bh + 1]) - 1;
  if (n <= 0) {
    write_neutral(pid, r, lane);
    return;
  }
  Stream sm;
  sm.u = 0, sm.u1 = (n + UT - 1) / UT;
  sm.s = 0;
  sm.cls = 2, sm.ntok = n, sm.blk0 = bh * kp->app_blocks, sm.nblk = kp->app_blocks, sm.gu0 = 0;
  sm.qrow = (bh / kp->num_kv_heads) * kp->num_q_heads + (bh % kp->num_kv_heads) * kp->rep;
  sm.pid = pid;
  sm.last_seg = -1;
  sm.ngran = 0, sm.nps = 0, sm.pseg0 = 0, sm.rank = 0, sm.counter = 0;
  sm.pi = -1, sm.p_unit0 = sm.p_nunits = sm.p_gran0 = sm.p_gran1 = sm.p_slot0 = 0;
  sm.tk0 = sm.tk1 = 0, sm.used = 0;
  sm.phase = 0;
  Piece cur = sm.next(lane);
  if (cur.nu > 0) run_class<HalfClass<G>, 2, G, AUX>(sm, cur, red, r, lane, true);
}

// One workgroup per worker; wave r of the workgroup serves query head r of every kv head it meets.
template <int G, int AUX>
__global__ __launch_bounds__(512) void decode_attention_kernel(DecodeParams) {
  extern __shared__ float red[];   // [rep][64][17] reduction tiles
  const int lane = threadIdx.x & 63;
  const int r = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // query head inside the group
#ifdef COCKTAIL_TRACE
  const uint64_t t_start = __builtin_amdgcn_s_memrealtime();
#endif
  if (int(blockIdx.x) >= kparams()->num_workers) {
    appended_tokens<G, AUX>(int(blockIdx.x) - kparams()->num_workers, red, r, lane);
    return;
  }
  Stream sm;
  sm.init(load_record(kparams()->recs + blockIdx.x));
  Piece cur = sm.next(lane);
  while (cur.nu > 0) {
    if (cur.cls == 0) {
      run_class<QuantClass<2, G>, 0, G, AUX>(sm, cur, red, r, lane);
    } else if (cur.cls == 1) {
      run_class<QuantClass<4, G>, 1, G, AUX>(sm, cur, red, r, lane);
    } else {
      run_class<HalfClass<G>, 2, G, AUX>(sm, cur, red, r, lane);
    }
  }
  // pool parts this worker never entered still own a partial slot: fill it with the neutral state
  for (int i = 0; i < sm.nps; ++i) {
    if ((sm.used >> i) & 1u) continue;
    const PoolSeg ps = load_record(kparams()->psegs + sm.pseg0 + i);
    if (sm.rank < ps.nslots) write_neutral(ps.slot0 + sm.rank, r, lane);
  }
#ifdef COCKTAIL_TRACE
  if (threadIdx.x == 0) {
    uint64_t* tr = kparams()->trace + blockIdx.x * 4;
    tr[0] = t_start;
    tr[1] = __builtin_amdgcn_s_memrealtime();
    tr[2] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | (31 << 11));    // HW_ID
    tr[3] = __builtin_amdgcn_s_getreg((20) | (0 << 6) | (31 << 11));   // XCC_ID
  }
#endif
}

// Exact merge of the partial states of one (sequence, query head):
//   M = max m_i,  L = sum l_i 2^(m_i - M),  out = sum o_i 2^(m_i - M) / L,  lse = ln2 (M + log2 L).
// The partials of a (sequence, kv head) are a dense block of the workspace.  512 threads: 32 channel
// quads x 16 slices of the block; a slice loads eight partials at a time (128 in flight per workgroup,
// usually the whole block in one round) and folds them with a running maximum, then the sixteen
// slice states are folded through shared memory.  A (sequence, query head) without any partial
// (empty sequence) gets zeros and lse = -inf.
constexpr int kMergeSlices = 16;
__global__ __launch_bounds__(32 * kMergeSlices) void decode_merge_kernel(DecodeParams prm) {
  __shared__ float sm_m[kMergeSlices];
  __shared__ float sm_l[kMergeSlices];
  __shared__ float sm_o[kMergeSlices][D];
  const int bhq = blockIdx.x;
  const int rep = prm.rep;
  const int b = bhq / prm.num_q_heads;
  const int hq = bhq - b * prm.num_q_heads;
  const int bh = b * prm.num_kv_heads + hq / rep;
  const int r = hq % rep;
  const int lo = prm.bh_off[bh];
  const int n = prm.bh_off[bh + 1] - lo;
  const int tid = threadIdx.x;
  // every worker has drawn its last ticket: put the counters back to zero for the next call
  if (blockIdx.x == 0)
    for (int i = tid; i < prm.num_groups; i += 32 * kMergeSlices) prm.counters[i * kCounterStride] = 0u;
  constexpr int STRIDE = D + kPartialFloats;
  constexpr int U = 8;   // partials in flight per thread
  const int quad = tid & 31, slice = tid >> 5;
  const float* base = prm.ws + (int64_t(lo) * rep + r) * STRIDE + kPartialFloats + quad * 4;
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
  for (int i0 = slice; i0 < n; i0 += kMergeSlices * U) {
    float pm[U], pl[U];
    float2 va[U], vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + kMergeSlices * u;
      const bool ok = i < n;
      const float* part = base + int64_t(ok ? i : i0) * rep * STRIDE;
      pm[u] = ok ? part[-kPartialFloats - quad * 4] : -INFINITY;
      pl[u] = part[1 - kPartialFloats - quad * 4];
      va[u] = *reinterpret_cast<const float2*>(part);
      vb[u] = *reinterpret_cast<const float2*>(part + 2);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float mn = fmaxf(m, pm[u]);
      // 2^(-inf - -inf) must not occur: a slice that has only seen padding keeps weight 0
      const float a = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mn);
      const float w = (pm[u] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(pm[u] - mn);
      l = l * a + pl[u] * w;
      o0 = o0 * a + va[u].x * w, o1 = o1 * a + va[u].y * w;
      o2 = o2 * a + vb[u].x * w, o3 = o3 * a + vb[u].y * w;
      m = mn;
    }
  }
  sm_o[slice][quad * 4 + 0] = o0, sm_o[slice][quad * 4 + 1] = o1;
  sm_o[slice][quad * 4 + 2] = o2, sm_o[slice][quad * 4 + 3] = o3;
  if (quad == 0) sm_m[slice] = m, sm_l[slice] = l;
  __syncthreads();
  if (tid < D) {
    float mx = sm_m[0];
#pragma unroll
    for (int sidx = 1; sidx < kMergeSlices; ++sidx) mx = fmaxf(mx, sm_m[sidx]);
    float big_l = 0.f, o = 0.f;
#pragma unroll
    for (int sidx = 0; sidx < kMergeSlices; ++sidx) {
      const float w = (sm_m[sidx] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[sidx] - mx);
      big_l += sm_l[sidx] * w;
      o += sm_o[sidx][tid] * w;
    }
    const bool empty = !(big_l > 0.f);
    prm.out[int64_t(bhq) * D + tid] = static_cast<_Float16>(empty ? 0.f : o / big_l);
    if (prm.lse && tid == 0) prm.lse[bhq] = empty ? -INFINITY : (mx + log2f(big_l)) * 0.6931471805599453f;
  }
}

}  // namespace cocktail

using namespace cocktail;

extern "C" int cocktail_default_workers(const cocktail_shape* shape, int32_t* num_workers) {
  if (int rc = check_shape(shape)) return rc;
  if (!num_workers) return fail(COCKTAIL_EINVAL, "num_workers is NULL");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return fail(COCKTAIL_EHIP, "no HIP device available");
  }
  const int rep = shape->num_q_heads / shape->num_kv_heads;
  const int waves_per_cu = 8;   // two waves per SIMD at <= 256 VGPRs
  int per_cu = waves_per_cu / rep;
  if (per_cu < 1) per_cu = 1;
  *num_workers = prop.multiProcessorCount * per_cu;
  return COCKTAIL_OK;
}

extern "C" int cocktail_decode_attention(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                         float sm_scale, void* out, float* lse, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  if (int rc = check_shape(shape)) return rc;
  if (!q || !out || !workspace) return fail(COCKTAIL_EINVAL, "q, out and workspace must not be NULL");
  if (!cache || !cache->plan_host || !cache->plan_dev) return fail(COCKTAIL_EINVAL, "cache or its plan is NULL");
  const PlanHeader* hd = static_cast<const PlanHeader*>(cache->plan_host);
  if (hd->magic != kPlanMagic || hd->version != kPlanVersion)
    return fail(COCKTAIL_EINVAL, "plan_host is not a plan written by this library version");
  if (hd->batch != shape->batch || hd->num_kv_heads != shape->num_kv_heads || hd->head_dim != shape->head_dim ||
      hd->chunk_size != shape->chunk_size || hd->group_size != shape->group_size ||
      hd->num_q_heads != shape->num_q_heads)
    return fail(COCKTAIL_EINVAL, "plan was made for a different shape");
  if (shape->head_dim != D)
    return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 128, got %d", shape->head_dim);
  if (hd->rep > COCKTAIL_MAX_Q_PER_KV)
    return fail(COCKTAIL_EUNSUPPORTED, "Hq/Hkv = %d exceeds %d", hd->rep, COCKTAIL_MAX_Q_PER_KV);
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(workspace) |
       reinterpret_cast<uintptr_t>(cache->plan_dev)) & 15)
    return fail(COCKTAIL_EALIGN, "q, out, workspace and plan_dev must be 16-byte aligned");
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3)) return fail(COCKTAIL_EALIGN, "lse must be 4-byte aligned");
  if (workspace_bytes < static_cast<size_t>(hd->workspace_bytes))
    return fail(COCKTAIL_ENOSPACE, "workspace holds %zu bytes, %lld needed", workspace_bytes,
                (long long)hd->workspace_bytes);
  DecodeParams p;
  char* pd = static_cast<char*>(cache->plan_dev);
  p.recs = reinterpret_cast<const WorkerRec*>(pd + hd->off_worker_rec);
  p.segs = reinterpret_cast<const Segment*>(pd + hd->off_segments);
  p.psegs = reinterpret_cast<const PoolSeg*>(pd + hd->off_pool_seg);
  p.counters = reinterpret_cast<uint32_t*>(pd + hd->off_counters);
  p.num_groups = hd->num_groups;
  p.num_workers = hd->num_workers;
  p.k_app = p.v_app = nullptr;
  p.num_appended = 0, p.app_blocks = hd->append_blocks;
  if (hd->append_capacity > 0) {
    if (!cache->k_app || !cache->v_app) return fail(COCKTAIL_EINVAL, "the plan has append buffers but k_app or v_app is NULL");
    if ((reinterpret_cast<uintptr_t>(cache->k_app) | reinterpret_cast<uintptr_t>(cache->v_app)) & 15)
      return fail(COCKTAIL_EALIGN, "append buffers must be 16-byte aligned");
    if (cache->num_appended < 0 || cache->num_appended > hd->append_capacity)
      return fail(COCKTAIL_EINVAL, "num_appended %d outside [0, %d]", cache->num_appended, hd->append_capacity);
    p.k_app = static_cast<const char*>(cache->k_app), p.v_app = static_cast<const char*>(cache->v_app);
    p.num_appended = cache->num_appended;
  } else if (cache->num_appended != 0) {
    return fail(COCKTAIL_EINVAL, "num_appended is %d but the plan was made without append buffers", cache->num_appended);
  }
  p.bh_off = reinterpret_cast<const int32_t*>(pd + hd->off_bh_off);
  p.q = static_cast<const uint32_t*>(q);
  for (int c = 0; c < 3; ++c) {
    if (hd->class_bytes[c] > 0 && (!cache->k[c] || !cache->v[c]))
      return fail(COCKTAIL_EINVAL, "cache buffer of class %d is NULL", c);
    if ((reinterpret_cast<uintptr_t>(cache->k[c]) | reinterpret_cast<uintptr_t>(cache->v[c])) & 15)
      return fail(COCKTAIL_EALIGN, "cache buffers must be 16-byte aligned");
    p.k[c] = static_cast<const char*>(cache->k[c]);
    p.v[c] = static_cast<const char*>(cache->v[c]);
  }
  p.ws = static_cast<float*>(workspace);
  p.out = static_cast<_Float16*>(out);
  p.lse = lse;
  if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt(static_cast<float>(shape->head_dim));
  p.scale_log2 = sm_scale * 1.4426950408889634f;
  p.rep = hd->rep, p.num_q_heads = hd->num_q_heads, p.num_kv_heads = hd->num_kv_heads;
#ifdef COCKTAIL_TRACE
  // debugging builds only: the caller provides 32 bytes per worker behind the regular workspace
  p.trace = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + ((hd->workspace_bytes + 255) & ~int64_t(255)));
#endif
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int app_groups = hd->append_capacity > 0 ? hd->batch * hd->num_kv_heads : 0;
  if (hd->total_gblocks > 0 || app_groups > 0) {
    const dim3 grid(hd->num_workers + app_groups, 1, 1), block(64 * hd->rep, 1, 1);
    const size_t lds = size_t(hd->rep) * 64 * 17 * sizeof(float);
    // non-temporal K/V loads when nothing is read twice: one wave per workgroup, and a cache large enough
    // that it cannot stay in the memory-side cache from one call to the next
    static const int nt_override = [] {   // tuning aid, read once: COCKTAIL_NON_TEMPORAL=0 | 1
      const char* e = std::getenv("COCKTAIL_NON_TEMPORAL");
      return e ? (std::atoi(e) != 0 ? 1 : 0) : -1;
    }();
    const bool nt = nt_override >= 0 ? nt_override == 1 : (hd->rep == 1 && hd->packed_bytes >= kNonTemporalMinBytes);
    void (*kern)(DecodeParams) = nullptr;
    switch (shape->group_size) {
      case 32: kern = nt ? decode_attention_kernel<32, kAuxNonTemporal> : decode_attention_kernel<32, kAuxDefault>; break;
      case 64: kern = nt ? decode_attention_kernel<64, kAuxNonTemporal> : decode_attention_kernel<64, kAuxDefault>; break;
      default: kern = nt ? decode_attention_kernel<128, kAuxNonTemporal> : decode_attention_kernel<128, kAuxDefault>; break;
    }
    hipLaunchKernelGGL(kern, grid, block, lds, st, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_attention launch failed: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL(decode_merge_kernel, dim3(shape->batch * shape->num_q_heads), dim3(32 * kMergeSlices), 0, st, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_merge launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}

// Decode side of Alg. 1 (Sec. III-C): single-query attention over the INT2, INT4
// and FP16 classes of the packed cache.
//
// Design (gfx950, wave64):
//  * The packed cache of a layer is one long stream of 64-token blocks ordered by
//    (sequence, kv head, class, block).  The host planner cuts that stream into
//    `num_workers` contiguous ranges of equal bytes; workgroup w streams range w.
//    Every workgroup therefore moves the same number of bytes whatever the class
//    mix is, and a range that crosses a (sequence, head) boundary simply emits one
//    partial state per (sequence, head) it touches.
//  * Inside a wave, lane i owns token i of the current block.  The block layout
//    stores the j-th 16-byte piece of all 64 tokens contiguously, so every load is
//    one fully coalesced 1 KiB global_load_dwordx4 per wave and the q.k dot product
//    of a token never leaves its lane: the query sits in scalar registers and feeds
//    v_dot2 as the uniform operand.  No cross-lane traffic exists in the steady
//    state; lanes are merged only when a partial state is flushed.
//  * Codes are expanded without any conversion: a code field masked out of a
//    half-word IS an fp16 subnormal of value code * 2^(pos-24), which v_dot2_f32_f16
//    and v_fma_mix_f32 consume exactly; the power of two is folded into per-group
//    factors.  Dequantisation is folded too:
//      q.k^      = sum_g scale_g * (q.code)_g + zero_g * sum(q_g)
//      sum p v^  = sum_t (p_t scale_tg) code_t + sum_t p_t zero_tg
//  * Loads are software pipelined by hand: the V blocks of a sub-split are in flight
//    while its logits are computed, and the K blocks of the next sub-split while the
//    V blocks are accumulated.
//  * Softmax is online per lane (each lane is its own split): logits of J blocks,
//    one lazy rescale when the lane's reference maximum grows by more than 2^8,
//    then the V pass.  (m, l, o[D]) partials go to the workspace and a second small
//    kernel merges them exactly (the softmax-weighted sum does not depend on how
//    tokens are grouped, Eq. 4-5).
//  * Grouped-query attention: the Hq/Hkv query heads of a kv head run as separate
//    waves of one workgroup on the same blocks, so the second to last read hits cache.
#include <hip/hip_runtime.h>

#include <cmath>

#include "common.h"
#include "plan.h"

namespace cocktail {

constexpr int D = 128;
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleThreshold = 8.0f;   // log2 units
constexpr float kTwo24 = 16777216.0f;

typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;

struct DecodeParams {
  const void* plan;
  const uint32_t* q;        // fp16 [B][Hq][D] viewed as dwords
  const char* k[3];
  const char* v[3];
  float* ws;                // [num_partials][rep][D + 2]
  float scale_log2;         // sm_scale * log2(e)
};

// A run of blocks is addressed through a buffer resource: every load is
// buffer_load(resource, lane offset in a VGPR, block/piece offset in an SGPR), so a lane needs
// one address register for the whole kernel, and reads past `bytes` return zero instead of faulting.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const char* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 load16(rsrc_t rs, uint32_t voff, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
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

// Zero-instruction anchor: the value must exist in a VGPR at this point of the program order.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }

template <int G>
struct LaneState {
  float acc[D];        // sum_t p_t * (scale * code | value)
  float zacc[D / G];   // sum_t p_t * zero_tg
  float m, l;
};

// ---------------------------------------------------------------- quantised classes
// A word holds 32/BITS codes; even channels in the low half-word, odd ones in the high
// half-word.  Masking field k of both half-words of `w` or `w >> 8` leaves two fp16
// subnormals  code * 2^(BITS*k - 24)  for the channel pair (2f, 2f+1), f = 4*half + k
// (INT2) or 2*half + k (INT4).
template <int BITS, int G>
struct QuantClass {
  static constexpr int PIECES = D * BITS / 128;
  static constexpr int NG = D / G;
  static constexpr int CPW = 32 / BITS;             // channels per word
  static constexpr int NPOS = 8 / BITS;             // fields per byte: 4 (INT2) or 2 (INT4)
  static constexpr int ROWB = D * BITS / 8;
  static constexpr int BLOCKB = kTB * (ROWB + 4 * NG);
  static constexpr uint32_t MASK0 = (BITS == 2) ? 0x00030003u : 0x000F000Fu;

  struct Stage {              // one lane's share of one block of K or V
    u32x4 pc[PIECES];
    uint32_t meta[NG];
  };

  // `boff` = byte offset of the block inside the run, `lane16` = lane * 16
  __device__ static __forceinline__ void load(Stage& s, rsrc_t rs, uint32_t boff, uint32_t lane16) {
#pragma unroll
    for (int p = 0; p < PIECES; ++p) s.pc[p] = load16(rs, lane16, boff + p * (kTB * 16));
    const uint32_t moff = boff + kTB * ROWB;
    if constexpr (NG == 4) {
      const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rs, lane16, moff, 0);
      s.meta[0] = t.x, s.meta[1] = t.y, s.meta[2] = t.z, s.meta[3] = t.w;
    } else if constexpr (NG == 2) {
      const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, lane16 >> 1, moff, 0);
      s.meta[0] = t.x, s.meta[1] = t.y;
    } else {
      s.meta[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, lane16 >> 2, moff, 0);
    }
  }

  // logit (log2 units) of this lane's token
  __device__ static __forceinline__ float logit(const Stage& s, const uint32_t (&q)[D / 2],
                                                const float (&qsum)[NG], float scale_log2) {
    float ga[NG][NPOS];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int k = 0; k < NPOS; ++k) ga[g][k] = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; ++p)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int cb = (p * 4 + wi) * CPW;          // first channel of the word
        const uint32_t w0 = s.pc[p][wi];
        const uint32_t w1 = w0 >> 8;
#pragma unroll
        for (int k = 0; k < NPOS; ++k) {
          const uint32_t mask = MASK0 << (BITS * k);
          ga[cb / G][k] = dot2(q[cb / 2 + k], w0 & mask, ga[cb / G][k]);
          ga[cb / G][k] = dot2(q[cb / 2 + NPOS + k], w1 & mask, ga[cb / G][k]);
        }
        sched_fence();   // keeps the masked temporaries of one word from piling up across words
      }
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float t = ga[g][NPOS - 1];
#pragma unroll
      for (int k = NPOS - 2; k >= 0; --k) t = t * (1.0f / float(1 << BITS)) + ga[g][k];
      // t = sum_d q_d code_d * 2^-24
      const h2 mz = as_h2(s.meta[g]);
      sum += (static_cast<float>(mz.x) * kTwo24) * t + static_cast<float>(mz.y) * qsum[g];
    }
    return sum * scale_log2;
  }

  __device__ static __forceinline__ void accumulate(const Stage& s, float p, LaneState<G>& st) {
    float ps[NG][NPOS];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
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
    for (int p_ = 0; p_ < PIECES; ++p_)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int cb = (p_ * 4 + wi) * CPW;
        const uint32_t w0 = s.pc[p_][wi];
        const uint32_t w1 = w0 >> 8;
#pragma unroll
        for (int k = 0; k < NPOS; ++k) {
          const uint32_t mask = MASK0 << (BITS * k);
          const uint32_t x0 = w0 & mask, x1 = w1 & mask;
          const float f = ps[cb / G][k];
          st.acc[cb + 2 * k] = fma_lo(f, x0, st.acc[cb + 2 * k]);
          st.acc[cb + 2 * k + 1] = fma_hi(f, x0, st.acc[cb + 2 * k + 1]);
          st.acc[cb + 2 * (NPOS + k)] = fma_lo(f, x1, st.acc[cb + 2 * (NPOS + k)]);
          st.acc[cb + 2 * (NPOS + k) + 1] = fma_hi(f, x1, st.acc[cb + 2 * (NPOS + k) + 1]);
        }
        // Pin the word's accumulators here: without it the optimiser sinks all multiply-adds of a
        // stage below the unpacking of every word and the masked temporaries spill.
#pragma unroll
        for (int i = 0; i < CPW; ++i) pin(st.acc[cb + i]);
        sched_fence();
      }
  }
};

// One lazy-rescale step of a lane's online softmax followed by p_j = 2^(s_j - m).
template <int G, int J>
__device__ __forceinline__ void softmax_step(const float (&s)[J], float (&p)[J], LaneState<G>& st) {
  float smax = s[0];
#pragma unroll
  for (int jj = 1; jj < J; ++jj) smax = fmaxf(smax, s[jj]);
  // the reference maximum only moves when it is exceeded by more than 2^8
  const bool grow = smax > st.m + kRescaleThreshold;
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
    const float mnew = grow ? smax : st.m;
    const float alpha = __builtin_amdgcn_exp2f(st.m - mnew);
    st.m = mnew;
    st.l *= alpha;
#pragma unroll
    for (int d = 0; d < D; ++d) st.acc[d] *= alpha;
#pragma unroll
    for (int g = 0; g < D / G; ++g) st.zacc[g] *= alpha;
  }
#pragma unroll
  for (int jj = 0; jj < J; ++jj) {
    p[jj] = __builtin_amdgcn_exp2f(s[jj] - st.m);
    st.l += p[jj];
  }
}

// Process `nb` (>= 1) consecutive blocks of a quantised class; `valid` = valid tokens in
// that range (only the last block can be partial).  J register stages rotate between K and
// V: as soon as the logit of a K block has been computed its registers receive the V block
// of the same tokens, and as soon as that has been accumulated they receive the K block J
// positions further on.  Blocks past the range are replaced by the last one and masked, so
// the loop body has no branches around the loads.
template <class CLS, int G, int J>
__device__ __forceinline__ void process_quant(const char* kblk, const char* vblk, int nb, int valid, int lane,
                                              const uint32_t (&q)[D / 2], const float (&qsum)[D / G],
                                              float scale_log2, LaneState<G>& st) {
  typename CLS::Stage sg[J];
  const int last = nb - 1;
  const uint32_t lane16 = lane * 16u;
  const rsrc_t krs = make_rsrc(kblk, uint32_t(nb) * CLS::BLOCKB), vrs = make_rsrc(vblk, uint32_t(nb) * CLS::BLOCKB);
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::load(sg[jj], krs, uint32_t(min(jj, last)) * CLS::BLOCKB, lane16);
#pragma unroll 1
  for (int j0 = 0; j0 < nb; j0 += J) {
    float s[J], p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      const float t = CLS::logit(sg[jj], q, qsum, scale_log2);
      s[jj] = ((j0 + jj) * kTB + lane < valid) ? t : -INFINITY;
      sched_fence();
      CLS::load(sg[jj], vrs, uint32_t(min(j0 + jj, last)) * CLS::BLOCKB, lane16);
      sched_fence();
    }
    softmax_step<G, J>(s, p, st);
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      CLS::accumulate(sg[jj], p[jj], st);
      sched_fence();
      CLS::load(sg[jj], krs, uint32_t(min(j0 + J + jj, last)) * CLS::BLOCKB, lane16);
      sched_fence();
    }
  }
}

// ---------------------------------------------------------------------- FP16 class
// A block is 16 pieces of K and 16 of V per lane.  Two 8-piece buffers rotate:
// K.lo K.hi | V.lo V.hi | next K.lo ..., each refilled as soon as it has been consumed.
template <int G>
__device__ __forceinline__ void process_half(const char* kblk, const char* vblk, int nb, int valid, int lane,
                                             const uint32_t (&q)[D / 2], float scale_log2, LaneState<G>& st) {
  constexpr int BLOCKB = kTB * 2 * D;
  constexpr int HP = 8;   // pieces per buffer
  u32x4 a[HP], b[HP];
  const uint32_t lane16 = lane * 16u;
  const rsrc_t krs = make_rsrc(kblk, uint32_t(nb) * BLOCKB), vrs = make_rsrc(vblk, uint32_t(nb) * BLOCKB);
  auto fill = [&](u32x4 (&buf)[HP], rsrc_t rs, uint32_t boff, int half) {
#pragma unroll
    for (int p = 0; p < HP; ++p) buf[p] = load16(rs, lane16, boff + (half * HP + p) * (kTB * 16));
  };
  auto qk = [&](const u32x4 (&buf)[HP], int half, float& a0, float& a1) {
#pragma unroll
    for (int p = 0; p < HP; ++p) {
      const int qb = (half * HP + p) * 4;
      a0 = dot2(q[qb + 0], buf[p][0], a0);
      a1 = dot2(q[qb + 1], buf[p][1], a1);
      a0 = dot2(q[qb + 2], buf[p][2], a0);
      a1 = dot2(q[qb + 3], buf[p][3], a1);
    }
  };
  auto pv = [&](const u32x4 (&buf)[HP], int half, float p) {
#pragma unroll
    for (int pi = 0; pi < HP; ++pi)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int d = ((half * HP + pi) * 4 + wi) * 2;
        st.acc[d] = fma_lo(p, buf[pi][wi], st.acc[d]);
        st.acc[d + 1] = fma_hi(p, buf[pi][wi], st.acc[d + 1]);
      }
  };
  const int last = nb - 1;
  fill(a, krs, 0, 0);
  fill(b, krs, 0, 1);
#pragma unroll 1
  for (int j = 0; j < nb; ++j) {
    const uint32_t vb = uint32_t(j) * BLOCKB;
    const uint32_t kn = uint32_t(min(j + 1, last)) * BLOCKB;
    float a0 = 0.f, a1 = 0.f;
    qk(a, 0, a0, a1);
    sched_fence();
    fill(a, vrs, vb, 0);
    sched_fence();
    qk(b, 1, a0, a1);
    sched_fence();
    fill(b, vrs, vb, 1);
    sched_fence();
    float s[1], p[1];
    s[0] = (j * kTB + lane < valid) ? (a0 + a1) * scale_log2 : -INFINITY;
    softmax_step<G, 1>(s, p, st);
    pv(a, 0, p[0]);
    sched_fence();
    fill(a, krs, kn, 0);
    sched_fence();
    pv(b, 1, p[0]);
    sched_fence();
    fill(b, krs, kn, 1);
    sched_fence();
  }
}

template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void decode_partial_kernel(DecodeParams prm) {
  constexpr int NG = D / G;
  extern __shared__ float red[];   // [rep][64][17]: one 16-channel reduction tile per wave

  const PlanHeader* hd = static_cast<const PlanHeader*>(prm.plan);
  const int w = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int r = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // query head inside the group
  const int rep = hd->rep;
  const int32_t* wg = plan_array<int32_t>(prm.plan, hd->off_worker_gblk);
  int g = wg[w];
  const int g1 = wg[w + 1];
  if (g >= g1) return;
  int s = plan_array<int32_t>(prm.plan, hd->off_worker_seg)[w];
  int pid = plan_array<int32_t>(prm.plan, hd->off_worker_pid)[w];
  const Segment* segs = plan_array<Segment>(prm.plan, hd->off_segments);

  LaneState<G> st;
  uint32_t q[D / 2];
  float qsum[NG];
  int cur_bh = -1;

  auto reset = [&]() {
#pragma unroll
    for (int d = 0; d < D; ++d) st.acc[d] = 0.f;
#pragma unroll
    for (int gq = 0; gq < NG; ++gq) st.zacc[gq] = 0.f;
    st.m = kNegBig;
    st.l = 0.f;
  };

  auto flush = [&]() {
    // merge the 64 lane states: common maximum, then sums
    float mw = st.m;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
    const float f = __builtin_amdgcn_exp2f(st.m - mw);
    float lw = st.l * f;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
    float* out = prm.ws + (int64_t(pid) * rep + r) * (D + kPartialFloats);
    if (lane == 0) {
      out[0] = mw;
      out[1] = lw;
    }
    float(*tile)[17] = reinterpret_cast<float(*)[17]>(red + r * 64 * 17);
#pragma unroll
    for (int ch = 0; ch < D / 16; ++ch) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int c = 0; c < 16; ++c) {
        const int d = ch * 16 + c;
        tile[lane][c] = (st.acc[d] + st.zacc[d / G]) * f;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const int c = lane & 15, quarter = lane >> 4;
      float sum = 0.f;
#pragma unroll
      for (int row = 0; row < 16; ++row) sum += tile[quarter * 16 + row][c];
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      if (lane < 16) out[kPartialFloats + ch * 16 + c] = sum;
    }
  };

  while (g < g1) {
    const Segment sg = segs[s];
    if (sg.bh != cur_bh) {
      if (cur_bh >= 0) {
        flush();
        ++pid;
      }
      cur_bh = sg.bh;
      reset();
      const int hq = sg.h * rep + r;
      const_u32_ptr qp = (const_u32_ptr)(prm.q + (int64_t(sg.b) * hd->num_q_heads + hq) * (D / 2));
#pragma unroll
      for (int i = 0; i < D / 2; ++i) q[i] = qp[i];
#pragma unroll
      for (int gq = 0; gq < NG; ++gq) {
        float a = 0.f;
#pragma unroll
        for (int i = 0; i < G / 2; ++i) a = dot2(q[gq * (G / 2) + i], 0x3C003C00u, a);   // (1.0, 1.0)
        qsum[gq] = a;
      }
    }
    const int jb = g - sg.gblk0;
    const int je = min(sg.nblk, g1 - sg.gblk0);
    const int nb = je - jb;
    if (nb <= 0) break;   // cannot happen with a plan written by cocktail_plan; guarantees termination
    // valid tokens of this range: up to the end of the segment or of the range, whichever comes first
    const int valid = min(sg.ntok - jb * kTB, nb * kTB);
    const int64_t first = int64_t(sg.blk0 + jb);
    if (sg.cls == 0) {
      using C = QuantClass<2, G>;
      process_quant<C, G, 4>(prm.k[0] + first * C::BLOCKB, prm.v[0] + first * C::BLOCKB, nb, valid,
                                             lane, q, qsum, prm.scale_log2, st);
    } else if (sg.cls == 1) {
      using C = QuantClass<4, G>;
      process_quant<C, G, 2>(prm.k[1] + first * C::BLOCKB, prm.v[1] + first * C::BLOCKB, nb, valid, lane, q, qsum,
                             prm.scale_log2, st);
    } else {
      constexpr int BB = kTB * 2 * D;
      process_half<G>(prm.k[2] + first * BB, prm.v[2] + first * BB, nb, valid, lane, q, prm.scale_log2, st);
    }
    g = sg.gblk0 + je;
    ++s;
  }
  flush();
}

// Exact merge of the partial states of one (sequence, query head):
//   M = max m_i,  L = sum l_i 2^(m_i - M),  out = sum o_i 2^(m_i - M) / L.
// 256 threads: 32 channel quads x 8 slices of the partial list.
__global__ __launch_bounds__(256) void decode_merge_kernel(const void* plan, const float* ws, _Float16* out,
                                                           float* lse) {
  __shared__ float sm_max[4];
  __shared__ float sm_l[8];
  __shared__ float sm_o[8][D];
  const PlanHeader* hd = static_cast<const PlanHeader*>(plan);
  const int bhq = blockIdx.x;
  const int rep = hd->rep;
  const int b = bhq / hd->num_q_heads;
  const int hq = bhq - b * hd->num_q_heads;
  const int bh = b * hd->num_kv_heads + hq / rep;
  const int r = hq % rep;
  const int32_t* bh_pid = plan_array<int32_t>(plan, hd->off_bh_pid);
  const int p0 = bh_pid[bh], p1 = bh_pid[bh + 1];
  const int tid = threadIdx.x;
  constexpr int STRIDE = D + kPartialFloats;
  float mx = -INFINITY;
  for (int p = p0 + tid; p < p1; p += 256) mx = fmaxf(mx, ws[(int64_t(p) * rep + r) * STRIDE]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  if ((tid & 63) == 0) sm_max[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sm_max[0], sm_max[1]), fmaxf(sm_max[2], sm_max[3]));
  const int quad = tid & 31, slice = tid >> 5;
  float o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f, big_l = 0.f;
  for (int p = p0 + slice; p < p1; p += 8) {
    const float* part = ws + (int64_t(p) * rep + r) * STRIDE;
    const float wgt = __builtin_amdgcn_exp2f(part[0] - mx);
    big_l += part[1] * wgt;
    const float2 v0 = *reinterpret_cast<const float2*>(part + kPartialFloats + quad * 4);
    const float2 v1 = *reinterpret_cast<const float2*>(part + kPartialFloats + quad * 4 + 2);
    o0 += v0.x * wgt, o1 += v0.y * wgt, o2 += v1.x * wgt, o3 += v1.y * wgt;
  }
  sm_o[slice][quad * 4 + 0] = o0, sm_o[slice][quad * 4 + 1] = o1;
  sm_o[slice][quad * 4 + 2] = o2, sm_o[slice][quad * 4 + 3] = o3;
  if (quad == 0) sm_l[slice] = big_l;
  __syncthreads();
  if (tid < D) {
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int sidx = 0; sidx < 8; ++sidx) l += sm_l[sidx], o += sm_o[sidx][tid];
    const bool empty = !(l > 0.f);
    out[int64_t(bhq) * D + tid] = static_cast<_Float16>(empty ? 0.f : o / l);
    if (lse && tid == 0) lse[bhq] = empty ? -INFINITY : (mx + log2f(l)) * 0.6931471805599453f;
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
  const int waves_per_cu = 4;   // one wave per SIMD, 512 registers each
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
  p.plan = cache->plan_dev;
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
  if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt(static_cast<float>(shape->head_dim));
  p.scale_log2 = sm_scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (hd->total_gblocks > 0) {
    const dim3 grid(hd->num_workers, 1, 1), block(64 * hd->rep, 1, 1);
    const size_t lds = size_t(hd->rep) * 64 * 17 * sizeof(float);
    switch (shape->group_size) {
      case 32: hipLaunchKernelGGL(decode_partial_kernel<32>, grid, block, lds, st, p); break;
      case 64: hipLaunchKernelGGL(decode_partial_kernel<64>, grid, block, lds, st, p); break;
      default: hipLaunchKernelGGL(decode_partial_kernel<128>, grid, block, lds, st, p); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_partial launch failed: %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL(decode_merge_kernel, dim3(shape->batch * shape->num_q_heads), dim3(256), 0, st,
                     cache->plan_dev, static_cast<const float*>(workspace), static_cast<_Float16*>(out), lse);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_merge launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}

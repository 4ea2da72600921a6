// Internal: the grouped-query decode kernel as templates over head_dim; one translation unit per head_dim
// instantiates launch_decode_quads<HD>.
//
// Decode side of Alg. 1 (Sec. III-C) when 2 to 8 query heads share a kv head (grouped-query attention).
//
// One wave serves up to four query heads of its kv head (5 to 8 heads: two waves per workgroup, one per
// four heads), so with up to four heads every K/V byte is fetched and unpacked once.  The
// per-token work is a small dense contraction (4 heads x 128 channels), done with the 4x4x4 fp16 matrix
// instruction, which multiplies sixteen independent 4x4 blocks, one per quad of lanes:
//     D[i][j] += sum_k A[i][k] * B[k][j]     lane 4b+i holds row i of A, lane 4b+j column j of B and of D.
//  * q.k:   A = the query (row = head, k = four channels), B = the lane's own token (the same four
//           channels of its K row), so lane 4b+j receives the logits of its token for the four heads.
//           Code fields are masked out of the packed words and fed to the instruction as they are (an
//           fp16 subnormal of value code * 2^(pos-24)); the power of two that depends on the field
//           position is put on the query channels once per state, scale and zero are applied to the
//           per-group sums:  q.k^ = sum_g scale_g (q.code)_g + zero_g sum(q_g).
//  * p.V:   needs k = tokens, i.e. four tokens of one channel side by side in a lane.  That is the
//           token-quad form of V: lane 4b+j of a 32-token unit holds tokens 4b..4b+3 of 16 channels.
//           A = p_t * scale_tg (row = head, k = the quad's four tokens), B = masked code fields, one
//           instruction per channel and lane, 4 heads x 16 channels of accumulators per lane.
//           p lives in "lane = token, register = head" form after the softmax; one more matrix
//           instruction with B = identity turns it into "lane = head, register = token".
//  * p * scale has to fit fp16.  The reference m of a head's partial state (p = 2^(logit - m); any reference
//    gives the same merged result) is therefore not tied to the largest logit but to the largest
//    logit + e, e = binary exponent of the token's V scale: it is kept >= that sum - 15, so p * scale < 2^15,
//    and is raised to (new largest sum) - 11 when exceeded, so the largest products sit near 2^11 whatever
//    the magnitude of V, with some 25 binary orders of fp16 range below them.
// Everything else (work pieces, pools, register stages, buffer loads) is shared with the one-head kernel.
#pragma once
#include <hip/hip_runtime.h>

#include "decode_common.h"

namespace cocktail {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr float kTopExp = 15.0f;     // p * scale stays below 2^kTopExp (fp16 holds up to 2^16 - 32)
constexpr float kHeadroom = 4.0f;    // log2 units left to grow into when the reference is moved
#define COCKTAIL_ARG(...) __VA_ARGS__   // a template-id with commas as one macro argument
constexpr int kRedStride = 36;      // floats per lane in the reduction tile (32 + padding, 16-byte aligned rows)

__device__ __forceinline__ f4 mfma4(u32x2 a, u32x2 b, f4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(h4, a), __builtin_bit_cast(h4, b), c, 0, 0, 0);
}
__device__ __forceinline__ u32x2 to_h4(f4 x) {
  h4 v;
  v[0] = static_cast<_Float16>(x[0]), v[1] = static_cast<_Float16>(x[1]);
  v[2] = static_cast<_Float16>(x[2]), v[3] = static_cast<_Float16>(x[3]);
  return __builtin_bit_cast(u32x2, v);
}
__device__ __forceinline__ f4 splat(float x) {
  f4 v = {x, x, x, x};
  return v;
}
__device__ __forceinline__ float pick(f4 v, int i) { return i == 0 ? v[0] : i == 1 ? v[1] : i == 2 ? v[2] : v[3]; }
__device__ __forceinline__ uint32_t pk_mul(uint32_t a, uint32_t b) { return as_u32(as_h2(a) * as_h2(b)); }
__device__ __forceinline__ f4 shfl_xor4(f4 v, int o) {
  f4 r;
  r[0] = __shfl_xor(v[0], o), r[1] = __shfl_xor(v[1], o), r[2] = __shfl_xor(v[2], o), r[3] = __shfl_xor(v[3], o);
  return r;
}
__device__ __forceinline__ f4 max4(f4 a, f4 b) {
  f4 r;
  r[0] = fmaxf(a[0], b[0]), r[1] = fmaxf(a[1], b[1]), r[2] = fmaxf(a[2], b[2]), r[3] = fmaxf(a[3], b[3]);
  return r;
}

template <int NGH>
struct QuadState {
  f4 acc[16];      // lane 4b+j: sum_t p_t scale_t code_t for its e-th channel (e = 0..15), one component per head
  f4 zacc[NGH];    // lane = token: sum over its tokens of p_t zero_tg, per head
  f4 l;            // lane = token: sum over its tokens of p_t, per head
  f4 m;            // reference maximum per head, the same in every lane
};

// ---------------------------------------------------------------- quantised classes
template <int HD, int BITS, int G>
struct QuadQuant : QuantClass<HD, BITS, G> {
  typedef QuantClass<HD, BITS, G> Base;
  typedef typename Base::Stage Stage;
  static constexpr int PH = Base::PH, NGH = Base::NGH, GL = Base::GL, CPW = Base::CPW, NPOS = Base::NPOS;
  static constexpr uint32_t MASK0 = Base::MASK0;
  static constexpr int PER = 16 / BITS;   // values per half-word of a token-quad word

  // 2^-(BITS k) in both halves of a dword
  __device__ static constexpr uint32_t pos_factor(int k) {
    const uint32_t h = uint32_t(15 - BITS * k) << 10;
    return h | (h << 16);
  }
  // what the accumulator of the lane's e-th channel has to be multiplied with at the end
  __device__ static constexpr float fac(int e) {
    const int k = (e % PER) % NPOS;
    return float(1 << (24 - BITS * k));
  }

  // Turns the lane's 64 query channels (dwords = channel pairs in natural order) into the sixteen A
  // operands in the order logits() walks through a K stage, each channel scaled by 2^-(BITS k) of the
  // field position k it will meet.
  __device__ static __forceinline__ void arrange_q(const uint32_t (&qraw)[DH / 2], u32x2 (&qa)[16]) {
#pragma unroll
    for (int w = 0; w < PH * 4; ++w)
#pragma unroll
      for (int k = 0; k < NPOS; ++k) {
        const int cb2 = w * CPW / 2;
        u32x2 a;
        a.x = pk_mul(qraw[cb2 + k], pos_factor(k));
        a.y = pk_mul(qraw[cb2 + NPOS + k], pos_factor(k));
        qa[w * NPOS + k] = a;
      }
  }

  // this lane's half of q.k^ for the four heads (natural units, before the softmax scale)
  __device__ static __forceinline__ f4 logits(const Stage& s, const u32x2 (&qa)[16], const f4 (&qs)[NGH]) {
    f4 ga[2] = {splat(0.f), splat(0.f)};   // two independent chains: by group where a lane has two, else by word
#pragma unroll
    for (int p = 0; p < PH; ++p)
#pragma unroll
      for (int wi = 0; wi < 4; ++wi) {
        const int w = p * 4 + wi;
        const int chain = NGH == 2 ? (w * CPW) / GL : (wi & 1);
        const uint32_t w0 = s.pc[p][wi];
        const uint32_t w1 = w0 >> 8;
#pragma unroll
        for (int k = 0; k < NPOS; ++k) {
          const uint32_t mask = MASK0 << (BITS * k);
          u32x2 b;
          b.x = w0 & mask, b.y = w1 & mask;
          ga[chain] = mfma4(qa[w * NPOS + k], b, ga[chain]);
        }
      }
    f4 sum;
    if constexpr (NGH == 2) {
      const h2 m0 = as_h2(s.meta[0]), m1 = as_h2(s.meta[1]);
      sum = (static_cast<float>(m0.x) * kTwo24) * ga[0] + static_cast<float>(m0.y) * qs[0];
      sum += (static_cast<float>(m1.x) * kTwo24) * ga[1] + static_cast<float>(m1.y) * qs[1];
    } else {
      const h2 m0 = as_h2(s.meta[0]);
      sum = (static_cast<float>(m0.x) * kTwo24) * (ga[0] + ga[1]) + static_cast<float>(m0.y) * qs[0];
    }
    return sum;
  }

  // binary exponent e of this lane's V scales: every scale is below 2^e
  __device__ static __forceinline__ float scale_exponent(const Stage& s) {
    int e = __builtin_amdgcn_frexp_expf(static_cast<float>(as_h2(s.meta[0]).x));
    if constexpr (NGH == 2) e = max(e, __builtin_amdgcn_frexp_expf(static_cast<float>(as_h2(s.meta[1]).x)));
    return static_cast<float>(e);
  }

  // p: the softmax weights of this lane's token for the four heads
  __device__ static __forceinline__ void accumulate(const Stage& s, f4 p, QuadState<NGH>& st, u32x2 ident) {
    u32x2 pa[NGH];   // lane = head: p_t scale_tg of the quad's four tokens
    // The weights go to the matrix unit rounded to fp16: x -> xr.  sum_t xr_t code_t is off by
    // sum_t (xr_t - x_t) code_t; adding c0 sum_t (x_t - xr_t), a constant per group like the zero term, leaves
    // sum_t (xr_t - x_t)(code_t - c0), and c0 = qmax / 2 centres the codes, which halves the bound.
    constexpr float c0 = 0.5f * float((1 << BITS) - 1);
#pragma unroll
    for (int g = 0; g < NGH; ++g) {
      const h2 mz = as_h2(s.meta[g]);
      const float sc = static_cast<float>(mz.x);
      const u32x2 x16 = to_h4(sc * p);
      const h2 r01 = as_h2(x16.x), r23 = as_h2(x16.y);
      // zero_t p_t + c0 (x_t - xr_t) with x_t = scale_t p_t:  (zero_t + c0 scale_t) p_t - c0 xr_t
      st.zacc[g] += (static_cast<float>(mz.y) + c0 * sc) * p;
      st.zacc[g][0] -= c0 * static_cast<float>(r01.x), st.zacc[g][1] -= c0 * static_cast<float>(r01.y);
      st.zacc[g][2] -= c0 * static_cast<float>(r23.x), st.zacc[g][3] -= c0 * static_cast<float>(r23.y);
      pa[g] = to_h4(mfma4(x16, ident, splat(0.f)));
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int wq = e / PER, f = e % PER, hi = f / NPOS, k = f % NPOS;
      const uint32_t wa = s.pc[(2 * wq) / 4][(2 * wq) % 4], wb = s.pc[(2 * wq + 1) / 4][(2 * wq + 1) % 4];
      const uint32_t mask = MASK0 << (BITS * k);
      u32x2 b;
      b.x = (hi ? wa >> 8 : wa) & mask, b.y = (hi ? wb >> 8 : wb) & mask;
      st.acc[e] = mfma4(pa[(32 * (e >> 3)) / GL], b, st.acc[e]);
    }
  }
};

// ---------------------------------------------------------------------- FP16 class
template <int HD, int G>
struct QuadHalf : HalfClass<HD, G> {
  typedef HalfClass<HD, G> Base;
  typedef typename Base::Stage Stage;
  static constexpr int NGH = Base::NGH;
  __device__ static constexpr float fac(int) { return 1.0f; }

  __device__ static __forceinline__ void arrange_q(const uint32_t (&qraw)[DH / 2], u32x2 (&qa)[16]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      u32x2 a;
      a.x = qraw[2 * i], a.y = qraw[2 * i + 1];
      qa[i] = a;
    }
  }

  __device__ static __forceinline__ f4 logits(const Stage& s, const u32x2 (&qa)[16], const f4 (&)[NGH]) {
    f4 ga[2] = {splat(0.f), splat(0.f)};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      u32x2 b;
      b.x = s.pc[i >> 1][2 * (i & 1)], b.y = s.pc[i >> 1][2 * (i & 1) + 1];
      ga[i & 1] = mfma4(qa[i], b, ga[i & 1]);
    }
    return ga[0] + ga[1];
  }

  __device__ static __forceinline__ float scale_exponent(const Stage&) { return 0.f; }   // raw values: p itself is the fp16 operand

  __device__ static __forceinline__ void accumulate(const Stage& s, f4 p, QuadState<NGH>& st, u32x2 ident) {
    const u32x2 pa = to_h4(mfma4(to_h4(p), ident, splat(0.f)));
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      u32x2 b;
      b.x = s.pc[e >> 1][2 * (e & 1)], b.y = s.pc[e >> 1][2 * (e & 1) + 1];
      st.acc[e] = mfma4(pa, b, st.acc[e]);
    }
  }
};

// Online softmax over the J units of one iteration, four heads at a time.  ev[jj]: exponent of the V scales
// of this lane's token in unit jj (see the note on the reference at the top).
template <int NGH, int J>
__device__ __forceinline__ void softmax_quads(const f4 (&s)[J], const float (&ev)[J], f4 (&p)[J], QuadState<NGH>& st) {
  f4 tmax = s[0] + ev[0];
#pragma unroll
  for (int jj = 1; jj < J; ++jj) tmax = max4(tmax, s[jj] + ev[jj]);
  const bool grow = tmax[0] > st.m[0] + kTopExp || tmax[1] > st.m[1] + kTopExp || tmax[2] > st.m[2] + kTopExp ||
                    tmax[3] > st.m[3] + kTopExp;
  if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) tmax = max4(tmax, shfl_xor4(tmax, o));
    f4 alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float mnew = tmax[i] > st.m[i] + kTopExp ? tmax[i] - (kTopExp - kHeadroom) : st.m[i];
      alpha[i] = __builtin_amdgcn_exp2f(st.m[i] - mnew);
      st.m[i] = mnew;
    }
    st.l *= alpha;
#pragma unroll
    for (int g = 0; g < NGH; ++g) st.zacc[g] *= alpha;
#pragma unroll
    for (int e = 0; e < 16; ++e) st.acc[e] *= alpha;
  }
#pragma unroll
  for (int jj = 0; jj < J; ++jj) {
#pragma unroll
    for (int i = 0; i < 4; ++i) p[jj][i] = __builtin_amdgcn_exp2f(s[jj][i] - st.m[i]);
    st.l += p[jj];
  }
}

// Writes the partial states `pid` of the wave's query heads: (m, l, o[HD]) per head, reduced over the lanes.
template <int HD, class CLS, int NGH, int GL>
__device__ __forceinline__ void flush_quads(const QuadState<NGH>& st, float* red, int pid, int r, int lane, int tokens) {
  constexpr int UT = Geo<HD>::UT;
  kparams_t prm = kparams();
  const int rep = prm->rep;
  const int heads = min(4, rep - 4 * r);   // query heads this wave really has
  // quantities kept per token lane: add up the lanes that hold different tokens (at head_dim 128 the 32 lanes
  // of each half; both halves hold the same p)
  f4 l = st.l;
  f4 z[NGH];
#pragma unroll
  for (int g = 0; g < NGH; ++g) z[g] = st.zacc[g];
#pragma unroll
  for (int o = UT / 2; o > 0; o >>= 1) {
    l += shfl_xor4(l, o);
#pragma unroll
    for (int g = 0; g < NGH; ++g) z[g] += shfl_xor4(z[g], o);
  }
  constexpr int STRIDE = HD + kPartialFloats;
  float* out = prm->ws + (int64_t(pid) * rep + 4 * r) * STRIDE;
  if (lane < heads) {
    out[lane * STRIDE] = pick(st.m, lane);
    out[lane * STRIDE + 1] = pick(l, lane);
    out[lane * STRIDE + 2] = __int_as_float(tokens);
  }
  // channel accumulators: lane 32h + 4b + j holds the sum over the tokens of quad b for 16 channels of half h
  // (head_dim 64: one half, sixteen quads over the 64 lanes); the quads are added through a shared-memory
  // tile, eight of the sixteen channels at a time.
  // Reader lane (h, head i, x) adds up, for j = 0..3, channel 64h + 32ps + 8j + x of head i.
  constexpr int NQ = UT / 4;   // token quads per unit
  const int hh = HD == 64 ? 0 : lane >> 5, ii = (lane >> 3) & 3, xx = lane & 7;
  const bool reader = HD == 128 || lane < 32;
#pragma unroll
  for (int ps = 0; ps < 2; ++ps) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int e8 = 0; e8 < 8; ++e8)
      *reinterpret_cast<f4*>(red + lane * kRedStride + e8 * 4) = st.acc[ps * 8 + e8] * CLS::fac(ps * 8 + e8);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float zv = pick(z[(32 * ps) / GL < NGH ? (32 * ps) / GL : 0], ii);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float sum = 0.f;
#pragma unroll
      for (int b = 0; b < NQ; ++b) sum += red[(32 * hh + 4 * b + j) * kRedStride + xx * 4 + ii];
      if (reader && ii < heads) out[ii * STRIDE + kPartialFloats + 64 * hh + 32 * ps + 8 * j + xx] = sum + zv;
    }
  }
}

// Zeroes the partial state, loads the query rows (lane 4b+i: its half of head i) and prepares the operands.
template <int HD, class CLS, int NGH, int GL>
__device__ __forceinline__ void begin_quads(int qrow, int h, int r, int lane, QuadState<NGH>& st,
                                            u32x2 (&qa)[16], f4 (&qs)[NGH]) {
#pragma unroll
  for (int e = 0; e < 16; ++e) st.acc[e] = splat(0.f);
#pragma unroll
  for (int g = 0; g < NGH; ++g) st.zacc[g] = splat(0.f), qs[g] = splat(0.f);
  st.l = splat(0.f);
  st.m = splat(kNegBig);
  const int rep = kparams()->rep;
  const int head = 4 * r + (lane & 3);   // wave r of the workgroup serves query heads 4r .. 4r+3 of the kv head
  const bool real = head < rep;   // rows of heads that do not exist are zero: their logits are 0, their output is dropped
  const u32x4* qp =
      reinterpret_cast<const u32x4*>(kparams()->q + int64_t(qrow + (real ? head : 0)) * (HD / 2) + h * (DH / 2));
  uint32_t qraw[DH / 2];
#pragma unroll
  for (int i = 0; i < DH / 8; ++i) {
    const u32x4 v = qp[i];
    qraw[4 * i] = real ? v.x : 0u, qraw[4 * i + 1] = real ? v.y : 0u;
    qraw[4 * i + 2] = real ? v.z : 0u, qraw[4 * i + 3] = real ? v.w : 0u;
  }
  // sum of the query channels per group and head, needed for the zero term: a product with a matrix of ones
  u32x2 ones;
  ones.x = ones.y = 0x3C003C00u;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    u32x2 a;
    a.x = qraw[2 * i], a.y = qraw[2 * i + 1];
    qs[(4 * i) / GL] = mfma4(a, ones, qs[(4 * i) / GL]);
  }
  CLS::arrange_q(qraw, qa);
}

// The quad kernel's version of the one-head kernel's run_class: same pipeline, four heads per wave.
template <int HD, class CLS, int CID, int G, int AUX>
__device__ __forceinline__ void run_quads(Stream<HD>& sm, Piece& cur, float* red, int r, int lane, bool app = false) {
  constexpr int NGH = CLS::NGH;
  constexpr int GL = G < DH ? G : DH;
  constexpr int J = CLS::J;
  constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  static_assert(J == kIterUnits[CID], "the planner cuts pool pieces to the kernel's iteration size");
  const int t = lane % UT, h = lane / UT;
  const uint32_t vc = CLS::code_voff(t, h), vm = CLS::meta_voff(t, h);
  const char* const kbase = uni(app ? kparams()->k_app : kparams()->k[CID]);
  const char* const vbase = uni(app ? kparams()->v_app : kparams()->v[CID]);
  const float scale_log2 = kparams()->scale_log2;
  u32x2 ident;   // column j of the 4x4 identity, j = lane % 4
  ident.x = (lane & 2) ? 0u : ((lane & 1) ? 0x3C000000u : 0x00003C00u);
  ident.y = (lane & 2) ? ((lane & 1) ? 0x3C000000u : 0x00003C00u) : 0u;
  QuadState<NGH> st;
  u32x2 qa[16];
  f4 qs[NGH];
  typename CLS::Stage ks[J], vs[J];
  int pid = cur.pid;
  rsrc_t krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  rsrc_t vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
  int ru = cur.us, rn = cur.nu;
  int roob = UPB * sm.nblk;
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
#pragma unroll
  for (int jj = 0; jj < J; ++jj) CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
  sched_fence();
  begin_quads<HD, CLS, NGH, GL>(sm.qrow, h, r, lane, st, qa, qs);
  int valid = cur.valid;
  int covered = 0;   // tokens the current partial states cover
  Piece nxt = sm.next(lane);
#pragma unroll 1
  while (true) {
    const bool more = nxt.nu > 0 && nxt.cls == CID;
    if (more) {
      krs = make_rsrc(kbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      vrs = make_rsrc(vbase + int64_t(sm.blk0) * CLS::BLOCKB, uint32_t(sm.nblk) * CLS::BLOCKB);
      ru = nxt.us, rn = nxt.nu, roob = UPB * sm.nblk;
    } else {
      rn = 0;
    }
    covered += valid;
    f4 s[J], p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      s[jj] = CLS::logits(ks[jj], qa, qs);
      sched_fence();
      CLS::template load<AUX>(ks[jj], krs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      f4 full = s[jj];
      if constexpr (HD == 128) full += shfl_xor4(s[jj], 32);   // both halves of the token
      full *= scale_log2;
      s[jj] = (jj * UT + t < valid) ? full : splat(-INFINITY);
    }
    float ev[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) ev[jj] = CLS::scale_exponent(vs[jj]);
    softmax_quads<NGH, J>(s, ev, p, st);
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      CLS::accumulate(vs[jj], p[jj], st, ident);
      sched_fence();
      CLS::template load<AUX>(vs[jj], vrs, jj < rn ? ru + jj : roob, vc, vm);
      sched_fence();
    }
    if (!more || nxt.fresh) flush_quads<HD, CLS, NGH, GL>(st, red, pid, r, lane, covered);
    if (!more) break;
    if (nxt.fresh) {
      pid = nxt.pid;
      covered = 0;
      begin_quads<HD, CLS, NGH, GL>(sm.qrow, h, r, lane, st, qa, qs);
    }
    valid = nxt.valid;
    nxt = sm.next(lane);
  }
  cur = nxt;
}

// Bytes of one stage buffer in shared memory: the K (or V) units of one loop iteration, the largest class counts.
constexpr int kStageBytes = 8 * 1024;
static_assert(J2 * (1024 + 512) <= kStageBytes && J4 * (2048 + 512) <= kStageBytes && J8 * (4096 + 512) <= kStageBytes &&
              J16 * 8192 <= kStageBytes, "a stage buffer holds the units of one iteration of every class");

// run_quads for workgroups of two waves (5 to 8 query heads of a kv head): both waves work on the same pieces,
// wave r for heads 4r .. 4r+3.  The K and V units are fetched once per workgroup, straight into shared memory
// (wave 0 fetches the K units of a piece, wave 1 its V units), into one of kStageSets sets of buffers; each wave
// reads its lanes' share from there, so nothing is fetched twice.  A second stream object runs kStageSets - 1
// pieces ahead of the one that drives the arithmetic and says what to fetch.  One workgroup barrier per iteration:
// after it the piece of this iteration is complete in its set and nobody reads the set of the piece before any
// more, so the next piece to fetch is sent there.  Both waves run the same scalar code on the same plan records
// (these workgroups take no pool tickets), hence the same sequence of barriers.  The reduction tile of a flush
// lives in the set that has just been used up, one wave after the other.
// Measured on MI355X (4 x 128K tokens, 64 query / 8 kv heads, 780 MB packed): two sets (32 KB of shared memory,
// four workgroups per compute unit) 200 us; three sets (48 KB, three workgroups) 242 us; both waves fetching
// everything for themselves into registers 210 us.  What counts is the number of resident waves: a wave's own
// instruction stream, not the bytes in flight, limits how fast a workgroup gets through its blocks.
#ifndef COCKTAIL_STAGE_SETS
#define COCKTAIL_STAGE_SETS 2
#endif
constexpr int kStageSets = COCKTAIL_STAGE_SETS;   // 2 or 3
constexpr int kAhead = kStageSets - 1;            // pieces that are fetched ahead of the one being worked on
// s_waitcnt vmcnt(NEWER): until all but the newest NEWER vector-memory operations of this wave are complete.
// Only vmcnt is waited for; the other counters get their maximum (expcnt 7, lgkmcnt 15).
template <int NEWER>
__device__ __forceinline__ void wait_all_but() {
  static_assert(NEWER >= 0 && NEWER < 16, "the low four bits of the count");
  __builtin_amdgcn_s_waitcnt(0x0F70 | NEWER);
}
template <int HD, class CLS, int CID, int G, int AUX>
__device__ __forceinline__ void run_quads_shared(Stream<HD>& sm, Piece& cur, char* stage, int r, int lane, bool app = false) {
  constexpr int NGH = CLS::NGH;
  constexpr int GL = G < DH ? G : DH;
  constexpr int J = CLS::J;
  constexpr int UT = Geo<HD>::UT, UPB = Geo<HD>::UPB;
  constexpr int UB = CLS::LDS_UNIT;
  constexpr int NI = J * (UB / 1024 + (UB % 1024) / 256);   // load instructions one wave issues per piece
  static_assert(J == kIterUnits[CID], "the planner cuts pool pieces to the kernel's iteration size");
  static_assert(J * UB <= kStageBytes, "stage buffer too small");
  const int t = lane % UT, h = lane / UT;
  const uint32_t vc = CLS::code_voff(t, h), vm = CLS::meta_voff(t, h);
  const char* const kbase = uni(app ? kparams()->k_app : kparams()->k[CID]);
  const char* const vbase = uni(app ? kparams()->v_app : kparams()->v[CID]);
  const float scale_log2 = kparams()->scale_log2;
  u32x2 ident;   // column j of the 4x4 identity, j = lane % 4
  ident.x = (lane & 2) ? 0u : ((lane & 1) ? 0x3C000000u : 0x00003C00u);
  ident.y = (lane & 2) ? ((lane & 1) ? 0x3C000000u : 0x00003C00u) : 0u;
  QuadState<NGH> st;
  u32x2 qa[16];
  f4 qs[NGH];
  int pid = cur.pid;
  // this wave fetches K (r = 0) or V (r = 1); buffer of (set, tensor x) at stage + (2 set + x) kStageBytes
  const char* const mybase = r == 0 ? kbase : vbase;
  auto fetch = [&](int set, const Stream<HD>& from, int ru, int rn) {   // `from` describes the segment of the piece
    const rsrc_t rs = make_rsrc(mybase + int64_t(from.blk0) * CLS::BLOCKB, uint32_t(from.nblk) * CLS::BLOCKB);
    lds_ptr_t dst = (lds_ptr_t)(stage + (2 * set + r) * kStageBytes);   // generic to shared: a C-style cast
    const int roob = UPB * from.nblk;
#pragma unroll
    for (int jj = 0; jj < J; ++jj) CLS::template load_lds<AUX>(dst + jj * UB, rs, jj < rn ? ru + jj : roob, vc, vm);
  };
  __syncthreads();   // the other wave may still be reading the buffers for the class that came before
  fetch(0, sm, cur.us, cur.nu);
  Stream<HD> ahead = sm;                     // the stream that says what to fetch: it runs ahead of `sm`
  Piece far;
  bool far_ok = true;
  if constexpr (kAhead == 2) {
    far = ahead.next(lane);                  // the piece after `cur`
    far_ok = far.nu > 0 && far.cls == CID;
    if (far_ok) fetch(1, ahead, far.us, far.nu);
  }
  begin_quads<HD, CLS, NGH, GL>(sm.qrow, h, r, lane, st, qa, qs);
  int valid = cur.valid;
  int covered = 0;   // tokens the current partial states cover
  int set = 0;
  Piece nxt = sm.next(lane);
#pragma unroll 1
  while (true) {
    const bool more = nxt.nu > 0 && nxt.cls == CID;
    // the piece to fetch now: kAhead pieces after the current one
    if (far_ok) {
      far = ahead.next(lane);
      far_ok = far.nu > 0 && far.cls == CID;
    }
    // this wave's fetches of the current piece have landed (with three sets those of the next one may still be on
    // their way: loads complete in order, and they are the newest NI of them)
    if (kAhead == 2 && more) wait_all_but<NI>();
    else wait_all_but<0>();
    __syncthreads();                 // ... and so have the other wave's; both are done with the set used before
    if (far_ok) fetch(set == 0 ? kStageSets - 1 : set - 1, ahead, far.us, far.nu);
    covered += valid;
    const char* const kst = stage + (2 * set) * kStageBytes;
    const char* const vst = kst + kStageBytes;
    f4 s[J], p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      typename CLS::Stage ks;
      CLS::read_lds(ks, kst + jj * UB, lane);
      s[jj] = CLS::logits(ks, qa, qs);
    }
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      f4 full = s[jj];
      if constexpr (HD == 128) full += shfl_xor4(s[jj], 32);   // both halves of the token
      full *= scale_log2;
      s[jj] = (jj * UT + t < valid) ? full : splat(-INFINITY);
    }
    typename CLS::Stage vs[J];
    float ev[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      CLS::read_lds(vs[jj], vst + jj * UB, lane);
      ev[jj] = CLS::scale_exponent(vs[jj]);
    }
    softmax_quads<NGH, J>(s, ev, p, st);
#pragma unroll
    for (int jj = 0; jj < J; ++jj) CLS::accumulate(vs[jj], p[jj], st, ident);
    if (!more || nxt.fresh) {
      // the set of this iteration is used up: it serves as the reduction tile, for one wave after the other
      float* tile = reinterpret_cast<float*>(stage + (2 * set) * kStageBytes);
      if (r == 0) flush_quads<HD, CLS, NGH, GL>(st, tile, pid, r, lane, covered);
      __syncthreads();
      if (r == 1) flush_quads<HD, CLS, NGH, GL>(st, tile, pid, r, lane, covered);
    }
    if (!more) break;
    if (nxt.fresh) {
      pid = nxt.pid;
      covered = 0;
      begin_quads<HD, CLS, NGH, GL>(sm.qrow, h, r, lane, st, qa, qs);
    }
    valid = nxt.valid;
    nxt = sm.next(lane);
    set = set == kStageSets - 1 ? 0 : set + 1;
  }
  cur = nxt;
}

// The neutral partial state for this wave's heads of a slot nobody had tokens for.
template <int HD>
__device__ __forceinline__ void write_neutral_heads(int slot, int r, int lane) {
  const int rep = kparams()->rep;
  for (int i = 4 * r; i < rep && i < 4 * r + 4; ++i) write_neutral<HD>(slot, i, lane);
}

template <int HD, int G, int AUX, int WAVES>
__device__ __forceinline__ void appended_tokens_quads(int idx, float* red, char* stage, int r, int lane) {
  const AppendSlice a = append_slice(idx);
  if (a.tokens <= 0) {
    write_neutral_heads<HD>(a.pid, r, lane);
    return;
  }
  Stream<HD> sm;
  sm.init_run(kFp16Class, a.tokens, a.first_block, a.blocks, a.qrow, a.pid);
  Piece cur = sm.next(lane);
  if (cur.nu > 0) {
    if constexpr (WAVES == 2) run_quads_shared<HD, QuadHalf<HD, G>, kFp16Class, G, AUX>(sm, cur, stage, r, lane, true);
    else run_quads<HD, QuadHalf<HD, G>, kFp16Class, G, AUX>(sm, cur, red, r, lane, true);
  }
}

// One workgroup per worker: one wave for 2 to 4 query heads per kv head, two waves (heads 0-3 and 4-7, both
// working on the same blocks, which they fetch once into shared memory: run_quads_shared) for 5 to 8.
template <int HD, int G, int AUX, int WAVES, bool INT8>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2))) void decode_quads_kernel(DecodeParams) {
  // one-wave workgroups: the reduction tile of a flush; two-wave workgroups: three sets of a K and a V buffer,
  // in which the tile finds its place too
  __shared__ __attribute__((aligned(16))) float red_all[WAVES == 2 ? 4 : 64 * kRedStride];
  __shared__ __attribute__((aligned(16))) char stage[WAVES == 2 ? kStageSets * 2 * kStageBytes : 16];
  static_assert(64 * kRedStride * sizeof(float) <= 2 * kStageBytes, "a set of stage buffers holds a reduction tile");
  const int lane = threadIdx.x & 63;
  const int r = WAVES == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* red = red_all;   // (not used by two-wave workgroups)
#ifdef COCKTAIL_TRACE
  const uint64_t t_start = __builtin_amdgcn_s_memrealtime();
#endif
  if (int(blockIdx.x) >= kparams()->num_workers) {
    appended_tokens_quads<HD, G, AUX, WAVES>(int(blockIdx.x) - kparams()->num_workers, red, stage, r, lane);
    return;
  }
  Stream<HD> sm;
  sm.init(load_record(kparams()->recs + blockIdx.x));
  // the two waves of a workgroup have to walk the same pieces (they meet at barriers): they take no pool tickets;
  // the planner gives such workgroups no pools (a plan that did would lose tokens, which the merge reports)
  if constexpr (WAVES == 2) sm.ngran = 0, sm.nps = 0;
  Piece cur = sm.next(lane);
  while (cur.nu > 0) {
#define COCKTAIL_RUN(CLS, CID)                                                                              \
  if constexpr (WAVES == 2) run_quads_shared<HD, CLS, CID, G, AUX>(sm, cur, stage, r, lane);              \
  else run_quads<HD, CLS, CID, G, AUX>(sm, cur, red, r, lane)
    if (cur.cls == 0) {
      COCKTAIL_RUN(COCKTAIL_ARG(QuadQuant<HD, 2, G>), 0);
    } else if (cur.cls == 1) {
      COCKTAIL_RUN(COCKTAIL_ARG(QuadQuant<HD, 4, G>), 1);
    } else if (INT8 && cur.cls == 2) {
      if constexpr (INT8) {
        COCKTAIL_RUN(COCKTAIL_ARG(QuadQuant<HD, 8, G>), 2);
      }
    } else {
      COCKTAIL_RUN(COCKTAIL_ARG(QuadHalf<HD, G>), kFp16Class);
    }
#undef COCKTAIL_RUN
  }
  for (int i = 0; i < sm.nps; ++i) {
    if ((sm.used >> i) & 1u) continue;
    const PoolSeg ps = load_record(kparams()->psegs + sm.pseg0 + i);
    if (sm.rank < ps.nslots) write_neutral_heads<HD>(ps.slot0 + sm.rank, r, lane);
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

template <int HD>
hipError_t launch_decode_quads(const DecodeParams& p, int group_size, bool non_temporal, bool int8, int grid, hipStream_t st) {
  const int waves = quad_waves(p.rep);
  void (*kern)(DecodeParams) = nullptr;
#define COCKTAIL_PICK2(G, I8) \
  kern = waves == 1 ? (non_temporal ? decode_quads_kernel<HD, G, kAuxNonTemporal, 1, I8> : decode_quads_kernel<HD, G, kAuxDefault, 1, I8>) \
                    : (non_temporal ? decode_quads_kernel<HD, G, kAuxNonTemporal, 2, I8> : decode_quads_kernel<HD, G, kAuxDefault, 2, I8>)
#define COCKTAIL_PICK(G)             \
  if (int8) COCKTAIL_PICK2(G, true); \
  else COCKTAIL_PICK2(G, false)
  if (group_size == 32) {
    COCKTAIL_PICK(32);
  } else if (group_size == 64) {
    COCKTAIL_PICK(64);
  } else if constexpr (HD >= 128) {
    COCKTAIL_PICK(128);
  }
#undef COCKTAIL_PICK
#undef COCKTAIL_PICK2
  if (!kern) return hipErrorInvalidValue;   // a group size larger than head_dim: refused by the shape check before
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * waves), 0, st, p);
  return hipGetLastError();
}

}  // namespace cocktail

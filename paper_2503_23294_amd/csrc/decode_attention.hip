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
//  * Codes are expanded with the fp16 "magic exponent" trick: (word & mask) | bias
//    is a pair of halves 2^k + code, the bias is removed exactly by one packed add.
//    Dequantisation is folded:  q.k^ = sum_g scale_g * (q.code)_g + zero_g * sum(q_g)
//    and  sum_t p_t v^_t = sum_t (p_t scale_tg) code_t + sum_t p_t zero_tg.
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

typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;

struct DecodeParams {
  const void* plan;
  const uint32_t* q;        // fp16 [B][Hq][D] viewed as dwords
  const char* k[3];
  const char* v[3];
  float* ws;                // [num_partials][rep][D + 2]
  float scale_log2;         // sm_scale * log2(e)
};

__device__ __forceinline__ u32x4 load16(const char* p) { return *reinterpret_cast<const u32x4*>(p); }

// (w & mask) | magic  ->  two halves 2^k + code ;  minus 2^k  ->  two halves holding the codes exactly
__device__ __forceinline__ h2 field(uint32_t w, uint32_t mask, uint32_t magic, float bias) {
  const uint32_t u = (w & mask) | magic;
  h2 b;
  b.x = static_cast<_Float16>(bias);
  b.y = b.x;
  return as_h2(u) - b;
}

// 16 two-bit codes of one word -> 8 half pairs (channel 2f, 2f+1 of the word)
__device__ __forceinline__ void unpack2(uint32_t w, h2 (&o)[8]) {
  const uint32_t t = w >> 10;
  o[0] = field(w, 0x00030003u, 0x64006400u, 1024.f);
  o[1] = field(w, 0x000C000Cu, 0x5C005C00u, 256.f);
  o[2] = field(w, 0x00300030u, 0x54005400u, 64.f);
  o[3] = field(w, 0x00C000C0u, 0x4C004C00u, 16.f);
  o[4] = field(w, 0x03000300u, 0x44004400u, 4.f);
  o[5] = field(t, 0x00030003u, 0x64006400u, 1024.f);
  o[6] = field(t, 0x000C000Cu, 0x5C005C00u, 256.f);
  o[7] = field(t, 0x00300030u, 0x54005400u, 64.f);
}

// 8 four-bit codes of one word -> 4 half pairs
__device__ __forceinline__ void unpack4(uint32_t w, h2 (&o)[4]) {
  const uint32_t t = w >> 8;
  o[0] = field(w, 0x000F000Fu, 0x64006400u, 1024.f);
  o[1] = field(w, 0x00F000F0u, 0x54005400u, 64.f);
  o[2] = field(t, 0x000F000Fu, 0x64006400u, 1024.f);
  o[3] = field(t, 0x00F000F0u, 0x54005400u, 64.f);
}

__device__ __forceinline__ float dot2(uint32_t qpair, h2 kv, float acc) {
  return __builtin_amdgcn_fdot2(as_h2(qpair), kv, acc, false);
}

template <int G>
struct LaneState {
  float acc[D];        // sum_t p_t * (scale * code | value)
  float zacc[D / G];   // sum_t p_t * zero_tg
  float m, l;
};

// ---------------------------------------------------------------- quantised classes
template <int BITS, int G>
struct QuantClass {
  static constexpr int PIECES = D * BITS / 128;
  static constexpr int NG = D / G;
  static constexpr int CPW = 32 / BITS;             // channels per word
  static constexpr int ROWB = D * BITS / 8;
  static constexpr int BLOCKB = kTB * (ROWB + 4 * NG);

  __device__ static __forceinline__ void load_meta(const char* blk, int lane, uint32_t (&meta)[NG]) {
    const char* mp = blk + kTB * ROWB + lane * (4 * NG);
    if constexpr (NG == 4) {
      const u32x4 t = *reinterpret_cast<const u32x4*>(mp);
      meta[0] = t.x, meta[1] = t.y, meta[2] = t.z, meta[3] = t.w;
    } else if constexpr (NG == 2) {
      const u32x2 t = *reinterpret_cast<const u32x2*>(mp);
      meta[0] = t.x, meta[1] = t.y;
    } else {
      meta[0] = *reinterpret_cast<const uint32_t*>(mp);
    }
  }

  // logit (log2 units) of this lane's token in block `blk`
  __device__ static __forceinline__ float logit(const char* blk, int lane, const uint32_t (&q)[D / 2],
                                                const float (&qsum)[NG], float scale_log2) {
    u32x4 pc[PIECES];
#pragma unroll
    for (int p = 0; p < PIECES; ++p) pc[p] = load16(blk + (p * kTB + lane) * 16);
    uint32_t meta[NG];
    load_meta(blk, lane, meta);
    float ga[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) ga[g] = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; ++p)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int word = p * 4 + k;
        const int cb = word * CPW;
        h2 c[CPW / 2];
        if constexpr (BITS == 2) unpack2(pc[p][k], c); else unpack4(pc[p][k], c);
#pragma unroll
        for (int f = 0; f < CPW / 2; ++f) ga[cb / G] = dot2(q[cb / 2 + f], c[f], ga[cb / G]);
      }
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const h2 mz = as_h2(meta[g]);
      s += static_cast<float>(mz.x) * ga[g] + static_cast<float>(mz.y) * qsum[g];
    }
    return s * scale_log2;
  }

  __device__ static __forceinline__ void accumulate(const char* blk, int lane, float p, LaneState<G>& st) {
    u32x4 pc[PIECES];
#pragma unroll
    for (int pi = 0; pi < PIECES; ++pi) pc[pi] = load16(blk + (pi * kTB + lane) * 16);
    uint32_t meta[NG];
    load_meta(blk, lane, meta);
    float ps[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const h2 mz = as_h2(meta[g]);
      ps[g] = p * static_cast<float>(mz.x);
      st.zacc[g] += p * static_cast<float>(mz.y);
    }
#pragma unroll
    for (int pi = 0; pi < PIECES; ++pi)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int cb = (pi * 4 + k) * CPW;
        h2 c[CPW / 2];
        if constexpr (BITS == 2) unpack2(pc[pi][k], c); else unpack4(pc[pi][k], c);
#pragma unroll
        for (int f = 0; f < CPW / 2; ++f) {
          st.acc[cb + 2 * f] += ps[cb / G] * static_cast<float>(c[f].x);
          st.acc[cb + 2 * f + 1] += ps[cb / G] * static_cast<float>(c[f].y);
        }
      }
  }
};

// ---------------------------------------------------------------------- FP16 class
template <int G>
struct HalfClass {
  static constexpr int PIECES = 16;
  static constexpr int BLOCKB = kTB * 2 * D;
  static constexpr int NG = D / G;

  __device__ static __forceinline__ float logit(const char* blk, int lane, const uint32_t (&q)[D / 2],
                                                const float (&)[NG], float scale_log2) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
      const u32x4 w = load16(blk + (p * kTB + lane) * 16);
      a0 = dot2(q[p * 4 + 0], as_h2(w.x), a0);
      a1 = dot2(q[p * 4 + 1], as_h2(w.y), a1);
      a0 = dot2(q[p * 4 + 2], as_h2(w.z), a0);
      a1 = dot2(q[p * 4 + 3], as_h2(w.w), a1);
    }
    return (a0 + a1) * scale_log2;
  }

  __device__ static __forceinline__ void accumulate(const char* blk, int lane, float p, LaneState<G>& st) {
#pragma unroll
    for (int pi = 0; pi < PIECES; ++pi) {
      const u32x4 w = load16(blk + (pi * kTB + lane) * 16);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const h2 v = as_h2(w[k]);
        st.acc[pi * 8 + 2 * k] += p * static_cast<float>(v.x);
        st.acc[pi * 8 + 2 * k + 1] += p * static_cast<float>(v.y);
      }
    }
  }
};

// Process `nb` consecutive blocks of one class starting at `blk` (K) / `vblk` (V);
// `valid` = number of valid tokens in that range (only the last block can be partial).
template <class CLS, int G, int J>
__device__ __forceinline__ void process_range(const char* kblk, const char* vblk, int nb, int valid, int lane,
                                              const uint32_t (&q)[D / 2], const float (&qsum)[D / G],
                                              float scale_log2, LaneState<G>& st) {
  for (int j0 = 0; j0 < nb; j0 += J) {
    float s[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      const int j = j0 + jj;
      s[jj] = -INFINITY;
      if (j < nb) {
        const float t = CLS::logit(kblk + int64_t(j) * CLS::BLOCKB, lane, q, qsum, scale_log2);
        if (j * kTB + lane < valid) s[jj] = t;
      }
    }
    float smax = s[0];
#pragma unroll
    for (int jj = 1; jj < J; ++jj) smax = fmaxf(smax, s[jj]);
    // lazy rescale: the reference maximum only moves when it is exceeded by more than 2^8
    const bool grow = smax > st.m + kRescaleThreshold;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      const float mnew = grow ? smax : st.m;
      const float alpha = __builtin_amdgcn_exp2f(st.m - mnew);
      st.m = mnew;
      st.l *= alpha;
#pragma unroll
      for (int d = 0; d < D; ++d) st.acc[d] *= alpha;
#pragma unroll
      for (int g = 0; g < D / G; ++g) st.zacc[g] *= alpha;
    }
    float p[J];
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      p[jj] = __builtin_amdgcn_exp2f(s[jj] - st.m);
      st.l += p[jj];
    }
#pragma unroll
    for (int jj = 0; jj < J; ++jj) {
      const int j = j0 + jj;
      if (j < nb) CLS::accumulate(vblk + int64_t(j) * CLS::BLOCKB, lane, p[jj], st);
    }
  }
}

template <int G>
__global__ __launch_bounds__(512) void decode_partial_kernel(DecodeParams prm) {
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
        h2 one;
        one.x = static_cast<_Float16>(1.0f);
        one.y = one.x;
#pragma unroll
        for (int i = 0; i < G / 2; ++i) a = dot2(q[gq * (G / 2) + i], one, a);
        qsum[gq] = a;
      }
    }
    const int jb = g - sg.gblk0;
    const int je = min(sg.nblk, g1 - sg.gblk0);
    const int nb = je - jb;
    if (nb <= 0) break;   // cannot happen with a plan written by cocktail_plan; guarantees termination
    const int valid = sg.ntok - jb * kTB;     // tokens from block jb to the end of the segment
    const int64_t first = int64_t(sg.blk0 + jb);
    if (sg.cls == 0) {
      using C = QuantClass<2, G>;
      process_range<C, G, 4>(prm.k[0] + first * C::BLOCKB, prm.v[0] + first * C::BLOCKB, nb, valid, lane, q, qsum,
                             prm.scale_log2, st);
    } else if (sg.cls == 1) {
      using C = QuantClass<4, G>;
      process_range<C, G, 2>(prm.k[1] + first * C::BLOCKB, prm.v[1] + first * C::BLOCKB, nb, valid, lane, q, qsum,
                             prm.scale_log2, st);
    } else {
      using C = HalfClass<G>;
      process_range<C, G, 1>(prm.k[2] + first * C::BLOCKB, prm.v[2] + first * C::BLOCKB, nb, valid, lane, q, qsum,
                             prm.scale_log2, st);
    }
    g = sg.gblk0 + je;
    ++s;
  }
  flush();
}

// Exact merge of the partial states of one (sequence, query head):
//   M = max m_i,  L = sum l_i 2^(m_i - M),  out = sum o_i 2^(m_i - M) / L.
__global__ __launch_bounds__(D) void decode_merge_kernel(const void* plan, const float* ws, _Float16* out,
                                                         float* lse) {
  const PlanHeader* hd = static_cast<const PlanHeader*>(plan);
  const int bhq = blockIdx.x;
  const int rep = hd->rep;
  const int b = bhq / hd->num_q_heads;
  const int hq = bhq - b * hd->num_q_heads;
  const int bh = b * hd->num_kv_heads + hq / rep;
  const int r = hq % rep;
  const int32_t* bh_pid = plan_array<int32_t>(plan, hd->off_bh_pid);
  const int p0 = bh_pid[bh], p1 = bh_pid[bh + 1];
  const int d = threadIdx.x;
  float mx = -INFINITY;
  for (int p = p0; p < p1; ++p) mx = fmaxf(mx, ws[(int64_t(p) * rep + r) * (D + kPartialFloats)]);
  float big_l = 0.f, o = 0.f;
  for (int p = p0; p < p1; ++p) {
    const float* part = ws + (int64_t(p) * rep + r) * (D + kPartialFloats);
    const float wgt = __builtin_amdgcn_exp2f(part[0] - mx);
    big_l += part[1] * wgt;
    o += part[kPartialFloats + d] * wgt;
  }
  const bool empty = !(big_l > 0.f);
  out[int64_t(bhq) * D + d] = static_cast<_Float16>(empty ? 0.f : o / big_l);
  if (lse && d == 0) lse[bhq] = empty ? -INFINITY : (mx + log2f(big_l)) * 0.6931471805599453f;
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
  if (shape->head_dim != D) return fail(COCKTAIL_EUNSUPPORTED, "kernels are built for head_dim 128, got %d", shape->head_dim);
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
  hipLaunchKernelGGL(decode_merge_kernel, dim3(shape->batch * shape->num_q_heads), dim3(D), 0, st, cache->plan_dev,
                     static_cast<const float*>(workspace), static_cast<_Float16*>(out), lse);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "decode_merge launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}
